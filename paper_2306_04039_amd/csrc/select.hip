// Final selection of stage 2 (Algorithm 1, last line): the k best of each query's scored candidates, returned
// best first under (score descending, item index ascending).
#include <math.h>

#include "common.hpp"
#include "msel.hpp"
#include "select.hpp"

namespace {

#define TOPK_MAX 1024

// ---- multi-workgroup form: three histogram passes, an emit pass into a k-slot staging list, a finishing sort -------
__global__ __launch_bounds__(MSEL_THREADS) void k_fin_hist(const float *scores, const int32_t *cand, int64_t Kp, int k,
                                                           uint32_t *mhist, int B, int pass) {
  __shared__ MselShared sh;
  const int b = blockIdx.y, blk = blockIdx.x, G = gridDim.x;
  uint32_t prefix = 0;
  if (pass > 0) {
    const MselCut c = msel_cut(mhist, B, b, (uint32_t)k, pass, sh);
    if (c.K == 0) return;
    prefix = c.prefix;
  }
  const float *sc = scores + (size_t)b * Kp;
  const int32_t *ci = cand ? cand + (size_t)b * Kp : nullptr;
  auto each = [&](auto f) {
    msel_slice_for_each<4>(sc, Kp, blk, G, [&](int64_t i, float v, bool valid) {
      if (valid) {
        const int32_t id = ci ? ci[i] : (int32_t)i;
        if (id >= 0) f(f32_to_key(v), (uint32_t)id);
      }
    });
  };
  msel_hist_pass(each, pass, prefix, mhist + ((size_t)pass * B + b) * MSEL_BINS, sh);
}

__global__ __launch_bounds__(MSEL_THREADS) void k_fin_emit(const float *scores, const int32_t *cand, int64_t Kp, int k,
                                                           const uint32_t *mhist, int B, uint32_t *mcnt,
                                                           uint32_t *tiebuf, uint2 *stage) {
  __shared__ MselShared sh;
  const int b = blockIdx.y, blk = blockIdx.x, G = gridDim.x;
  const MselCut c = msel_cut(mhist, B, b, (uint32_t)k, MSEL_PASSES, sh);
  if (c.K == 0) return;
  const uint32_t kth = c.prefix;
  const bool all_ties = (c.krem == c.cnt);
  const float *sc = scores + (size_t)b * Kp;
  const int32_t *ci = cand ? cand + (size_t)b * Kp : nullptr;
  uint32_t *mc = mcnt + (size_t)b * MCNT_STRIDE;
  msel_slice_for_each<4>(sc, Kp, blk, G, [&](int64_t i, float v, bool valid) {
    int32_t id = -1;
    if (valid) id = ci ? ci[i] : (int32_t)i;
    const uint32_t key = f32_to_key(v);
    const bool ok = valid && id >= 0;
    const bool at = ok && key == kth;
    const bool take = ok && (key > kth || (at && all_ties));
    const bool tie = at && !all_ties;
    if (__ballot(take)) {
      const uint32_t slot = msel_wave_slot(take, mc);
      if (take && slot < TOPK_MAX) stage[(size_t)b * TOPK_MAX + slot] = make_uint2(key, (uint32_t)id);
    }
    if (__ballot(tie)) {
      const uint32_t ts = msel_wave_slot(tie, mc + 1);
      if (tie && ts < MSEL_TIE_CAP) tiebuf[(size_t)b * MSEL_TIE_CAP + ts] = (uint32_t)id;
    }
  });
}

__global__ __launch_bounds__(MSEL_THREADS) void k_fin_finish(int k, const uint32_t *mhist, int B, uint32_t *mcnt,
                                                             const uint32_t *tiebuf, const uint2 *stage,
                                                             int32_t *out_idx, float *out_score) {
  __shared__ MselShared sh;
  __shared__ uint32_t skey[TOPK_MAX];
  __shared__ uint32_t sidx[TOPK_MAX];
  const int b = blockIdx.x, tid = threadIdx.x;
  const MselCut c = msel_cut(mhist, B, b, (uint32_t)k, MSEL_PASSES, sh);
  const uint32_t kk = c.K;  // number of real results
  for (int i = tid; i < TOPK_MAX; i += MSEL_THREADS) {
    skey[i] = 0u;  // sorts last
    sidx[i] = 0xffffffffu;
  }
  __syncthreads();
  if (kk > 0) {
    const bool partial_ties = (c.krem != c.cnt);
    if (partial_ties && c.cnt > MSEL_TIE_CAP) {
      if (tid == 0) mcnt[(size_t)b * MCNT_STRIDE + 2] = 1u;  // left to the single-workgroup selection
      return;
    }
    const uint32_t nabove = partial_ties ? kk - c.krem : kk;
    for (uint32_t i = tid; i < nabove; i += MSEL_THREADS) {
      const uint2 e = stage[(size_t)b * TOPK_MAX + i];
      skey[i] = e.x;
      sidx[i] = e.y;
    }
    __syncthreads();
    if (partial_ties)
      msel_take_lowest_ties(tiebuf + (size_t)b * MSEL_TIE_CAP, c.cnt, c.krem, sh, [&](uint32_t rank, uint32_t idx) {
        skey[nabove + rank] = c.prefix;
        sidx[nabove + rank] = idx;
      });
  }
  __syncthreads();
  // bitonic sort of the first `width` slots (the power of two covering k) by (key desc, idx asc)
  int width = 64;
  while (width < k) width <<= 1;
  for (int size = 2; size <= width; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int i = tid; i < width; i += MSEL_THREADS) {
        const int j = i ^ stride;
        if (j > i) {
          const uint32_t ki = skey[i], kj = skey[j], ii = sidx[i], ij = sidx[j];
          const bool i_first = ki > kj || (ki == kj && ii < ij);
          const bool up = ((i & size) == 0);
          if (up ? !i_first : i_first) {
            skey[i] = kj; skey[j] = ki;
            sidx[i] = ij; sidx[j] = ii;
          }
        }
      }
      __syncthreads();
    }
  }
  for (int i = tid; i < k; i += MSEL_THREADS) {
    const bool real = (uint32_t)i < kk;
    out_idx[(size_t)b * k + i] = real ? (int32_t)sidx[i] : -1;
    out_score[(size_t)b * k + i] = real ? key_to_f32(skey[i]) : -INFINITY;
  }
}

// ---- single-workgroup form: used only for queries with more than MSEL_TIE_CAP items tied at the k-th score ---------
__global__ __launch_bounds__(SELECT_THREADS) void k_final_topk(const float *scores, const int32_t *cand, int64_t Kp,
                                                               int k, const uint32_t *enable, int32_t *out_idx,
                                                               float *out_score) {
  __shared__ SelectShared sh;
  __shared__ uint32_t skey[TOPK_MAX];
  __shared__ uint32_t sidx[TOPK_MAX];
  __shared__ uint32_t nvalid_s;
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  if (enable && enable[(size_t)b * MCNT_STRIDE] == 0u) return;
  const float *sc = scores + (size_t)b * Kp;
  const int32_t *ci = cand ? cand + (size_t)b * Kp : nullptr;
  auto each = [&](auto f) {
    block_for_each<4>(sc, Kp, [&](int64_t i, float v) {
      const int32_t id = ci ? ci[i] : (int32_t)i;
      if (id >= 0) f(f32_to_key(v), (uint32_t)id);
    });
  };
  // number of valid candidates
  if (tid == 0) nvalid_s = 0;
  __syncthreads();
  uint32_t mine = 0;
  for (int64_t i = tid; i < Kp; i += SELECT_THREADS) mine += (ci ? ci[i] >= 0 : true) ? 1u : 0u;
  for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor((int)mine, o);
  if ((tid & 63) == 0 && mine) atomicAdd(&nvalid_s, mine);
  __syncthreads();
  const uint32_t nvalid = nvalid_s;
  const uint32_t kk = nvalid < (uint32_t)k ? nvalid : (uint32_t)k;  // how many real results
  for (int i = tid; i < TOPK_MAX; i += SELECT_THREADS) {
    skey[i] = 0u;            // sorts last
    sidx[i] = 0xffffffffu;
  }
  if (tid == 0) sh.out_count = 0;
  __syncthreads();
  if (kk > 0) {
    block_select_kth<true>(each, kk, sh);
    each([&](uint32_t key, uint32_t idx) {
      if (select_accept(key, idx, sh)) {
        uint32_t slot = atomicAdd(&sh.out_count, 1u);
        if (slot < TOPK_MAX) {
          skey[slot] = key;
          sidx[slot] = idx;
        }
      }
    });
  }
  __syncthreads();
  // bitonic sort of TOPK_MAX (key desc, idx asc); one element per thread
  for (int size = 2; size <= TOPK_MAX; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      const int i = tid, j = tid ^ stride;
      if (j > i) {
        const uint32_t ki = skey[i], kj = skey[j], ii = sidx[i], ij = sidx[j];
        const bool i_first = ki > kj || (ki == kj && ii < ij);  // i belongs before j in the final order
        const bool up = ((i & size) == 0);
        if (up ? !i_first : i_first) {
          skey[i] = kj; skey[j] = ki;
          sidx[i] = ij; sidx[j] = ii;
        }
      }
      __syncthreads();
    }
  }
  for (int i = tid; i < k; i += SELECT_THREADS) {
    const bool real = (uint32_t)i < kk;
    out_idx[(size_t)b * k + i] = real ? (int32_t)sidx[i] : -1;
    out_score[(size_t)b * k + i] = real ? key_to_f32(skey[i]) : -INFINITY;
  }
}

}  // namespace

size_t final_topk_workspace_bytes(int B) {
  size_t off = align_up((size_t)MSEL_PASSES * B * MSEL_BINS * 4 + (size_t)B * MCNT_STRIDE * 4, 256);
  off = align_up(off + (size_t)B * MSEL_TIE_CAP * 4, 256);
  off = align_up(off + (size_t)B * TOPK_MAX * 8, 256);
  return off;
}

mol_status_t launch_final_topk(const float *scores, const int32_t *cand_idx, int B, int64_t Kp, int k,
                               int32_t *out_idx, float *out_score, char *ws, hipStream_t st) {
  if (k > TOPK_MAX) return mol_fail(MOL_EUNSUPPORTED, "k=%d exceeds the supported maximum %d", k, TOPK_MAX);
  ProfScope ps(MOL_PROF_FINAL_TOPK, st);
  uint32_t *mhist = reinterpret_cast<uint32_t *>(ws);
  uint32_t *mcnt = mhist + (size_t)MSEL_PASSES * B * MSEL_BINS;
  size_t off = align_up((size_t)MSEL_PASSES * B * MSEL_BINS * 4 + (size_t)B * MCNT_STRIDE * 4, 256);
  uint32_t *tiebuf = reinterpret_cast<uint32_t *>(ws + off);
  off = align_up(off + (size_t)B * MSEL_TIE_CAP * 4, 256);
  uint2 *stage = reinterpret_cast<uint2 *>(ws + off);
  const size_t nz = (size_t)MSEL_PASSES * B * MSEL_BINS + (size_t)B * MCNT_STRIDE;
  hipLaunchKernelGGL(k_zero_u32, dim3((unsigned)((nz + 1023) / 1024)), dim3(256), 0, st, mhist, nz);
  HIP_TRY(hipGetLastError());
  int G = 512 / B;
  G = G < 1 ? 1 : (G > 32 ? 32 : G);
  const int64_t gmax = (Kp + 4 * MSEL_THREADS - 1) / (4 * MSEL_THREADS);
  if (G > gmax) G = (int)gmax;
  for (int pass = 0; pass < MSEL_PASSES; ++pass) {
    hipLaunchKernelGGL(k_fin_hist, dim3(G, B), dim3(MSEL_THREADS), 0, st, scores, cand_idx, Kp, k, mhist, B, pass);
    HIP_TRY(hipGetLastError());
  }
  hipLaunchKernelGGL(k_fin_emit, dim3(G, B), dim3(MSEL_THREADS), 0, st, scores, cand_idx, Kp, k, mhist, B, mcnt, tiebuf,
                     stage);
  HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(k_fin_finish, dim3(B), dim3(MSEL_THREADS), 0, st, k, mhist, B, mcnt, tiebuf, stage, out_idx,
                     out_score);
  HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(k_final_topk, dim3(B), dim3(SELECT_THREADS), 0, st, scores, cand_idx, Kp, k, mcnt + 2, out_idx,
                     out_score);
  HIP_TRY(hipGetLastError());
  return MOL_OK;
}
