// Final selection of stage 2 (Algorithm 1, last line): the k best of each query's scored candidates, returned
// best first under (score descending, item index ascending).
#include <math.h>

#include "common.hpp"
#include "select.hpp"

namespace {

#define TOPK_MAX 1024

// ---- level 1 of the two-level form: workgroup (g, b) keeps the k best of its slice of query b's row -------------------
// With k much smaller than the row (k = 100 of K' = 1e5) the k best of the row are among the k best of each of G slices,
// so G workgroups per query cut the row to G*k staged candidates in one pass over it, and one workgroup per query
// finishes.  Staged rows are (score, item index) pairs, unordered, padded with (-inf, -1).
// Long slices are cut first with a bound that cannot lose anything: the k-th best key of ANY subset of the slice is a
// lower bound of the slice's k-th best key, so after the k-th best of the slice's first eighth is known (the multi-pass
// radix selection, on an eighth of the data), ONE pass over the slice collects every entry that reaches it -- about 8 k
// of them when the slice is in no particular order -- into an LDS buffer, and the exact k best are selected there.
// When the buffer overflows (a slice sorted by score, masses of ties) the multi-pass selection runs on the whole slice.
#define SEG_PREFIX_MIN 4096  // shortest slice that takes the prefix-bound path
#define SEG_CAP 4096          // entries of the LDS buffer
__global__ __launch_bounds__(SELECT_THREADS) void k_seg_topk(const float *scores, const int32_t *cand,
                                                             const int32_t *cand_count, int64_t Kp, int k,
                                                             float *st_score, int32_t *st_idx) {
  __shared__ SelectShared sh;
  __shared__ uint2 s_buf[SEG_CAP];
  __shared__ uint32_t s_cnt;
  const int g = blockIdx.x, G = gridDim.x, b = blockIdx.y;
  const int tid = threadIdx.x;
  const int64_t per = (Kp + G - 1) / G;
  const int64_t lo = (int64_t)g * per;
  const int64_t row = (cand_count && cand_count[b] < Kp) ? (cand_count[b] < 0 ? 0 : cand_count[b]) : Kp;  // slots in use
  const int64_t n = lo >= row ? 0 : (lo + per <= row ? per : row - lo);
  const float *sc = scores + (size_t)b * Kp + lo;
  const int32_t *ci = cand ? cand + (size_t)b * Kp + lo : nullptr;
  float *os = st_score + ((size_t)b * G + g) * k;
  int32_t *oi = st_idx + ((size_t)b * G + g) * k;
  auto each_of = [&](int64_t len) {
    return [&, len](auto f) {
      block_for_each<4>(sc, len, [&](int64_t i, float v) {
        const int32_t id = ci ? ci[i] : (int32_t)(lo + i);
        if (id >= 0) f(f32_to_key(v), (uint32_t)id);
      });
    };
  };
  auto each = each_of(n);
  // writes the accepted entries of `from` (exactly kk of them, up to entries listed twice) and pads the rest
  auto emit = [&](auto from, uint32_t kk) {
    if (tid == 0) sh.out_count = 0;
    __syncthreads();
    if (kk > 0) {
      auto put = [&](uint32_t key, uint32_t idx) {
        const uint32_t slot = atomicAdd(&sh.out_count, 1u);
        if (slot < kk) {
          os[slot] = key_to_f32(key);
          oi[slot] = (int32_t)idx;
        }
      };
      from([&](uint32_t key, uint32_t idx) {
        if (select_before_kth(key, idx, sh)) put(key, idx);
      });
      if (sh.idx_limit != 0xffffffffu) {  // copies of the K-th element itself fill what is left
        __syncthreads();
        from([&](uint32_t key, uint32_t idx) {
          if (select_equals_kth(key, idx, sh)) put(key, idx);
        });
      }
    }
    for (uint32_t i = kk + tid; i < (uint32_t)k; i += SELECT_THREADS) {
      os[i] = -INFINITY;
      oi[i] = -1;
    }
  };

  if (n >= SEG_PREFIX_MIN) {
    auto each_prefix = each_of(n / 8);
    const uint32_t kp = block_select_kth<false, false>(each_prefix, (uint32_t)k, sh);  // k-th best key of the first eighth
    const uint32_t bound = (kp == (uint32_t)k) ? sh.kth_key : 0u;               // fewer than k valid entries there: no bound
    __syncthreads();
    if (tid == 0) s_cnt = 0;
    __syncthreads();
    each([&](uint32_t key, uint32_t idx) {
      if (key >= bound) {
        const uint32_t slot = atomicAdd(&s_cnt, 1u);
        if (slot < SEG_CAP) s_buf[slot] = make_uint2(key, idx);
      }
    });
    __syncthreads();
    const uint32_t cnt = s_cnt;
    if (cnt <= SEG_CAP) {  // the buffer holds every entry that can be among the k best (at least k of them, if k exist)
      auto each_buf = [&](auto f) {
        for (uint32_t e = tid; e < cnt; e += SELECT_THREADS) {
          const uint2 v = s_buf[e];
          f(v.x, v.y);
        }
      };
      const uint32_t kk = block_select_kth<true, false>(each_buf, (uint32_t)k, sh);
      emit(each_buf, kk);
      return;
    }
    __syncthreads();
  }

  const uint32_t kk = block_select_kth<true, false>(each, (uint32_t)k, sh);  // min(k, valid entries of the slice)
  emit(each, kk);
}

// ---- one workgroup per query: radix select of the k-th element, then a sort of the k winners -----------------------
#ifndef MOL_FINAL_PREFIX
#define MOL_FINAL_PREFIX 1
#endif
#define FINAL_PREFIX_MIN 8192  // shortest row that takes the prefix-bound path
__global__ __launch_bounds__(SELECT_THREADS) void k_final_topk(const float *scores, const int32_t *cand,
                                                               const int32_t *cand_count, int64_t Kp, int k, int nsort,
                                                               int32_t *out_idx, float *out_score) {
  __shared__ SelectShared sh;
  __shared__ uint32_t skey[TOPK_MAX];
  __shared__ uint32_t sidx[TOPK_MAX];
#if MOL_FINAL_PREFIX
  __shared__ uint2 s_buf[SEG_CAP];
  __shared__ uint32_t s_cnt;
#endif
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const float *sc = scores + (size_t)b * Kp;
  const int32_t *ci = cand ? cand + (size_t)b * Kp : nullptr;
  const int64_t row = (cand_count && cand_count[b] < Kp) ? (cand_count[b] < 0 ? 0 : cand_count[b]) : Kp;  // slots in use
  auto each = [&](auto f) {
    block_for_each<4>(sc, row, [&](int64_t i, float v) {
      const int32_t id = ci ? ci[i] : (int32_t)i;
      if (id >= 0) f(f32_to_key(v), (uint32_t)id);
    });
  };
  for (int i = tid; i < TOPK_MAX; i += SELECT_THREADS) {
    skey[i] = 0u;            // sorts last
    sidx[i] = 0xffffffffu;
  }
  if (tid == 0) sh.out_count = 0;
  // the accepted entries of `from` (kk of them) go to the sort buffer
  auto take = [&](auto from, uint32_t kk) {
    if (kk > 0) {
      auto put = [&](uint32_t key, uint32_t idx) {
        uint32_t slot = atomicAdd(&sh.out_count, 1u);
        if (slot < kk) {
          skey[slot] = key;
          sidx[slot] = idx;
        }
      };
      from([&](uint32_t key, uint32_t idx) {
        if (select_before_kth(key, idx, sh)) put(key, idx);
      });
      if (sh.idx_limit != 0xffffffffu) {  // copies of the K-th element itself fill what is left
        __syncthreads();
        from([&](uint32_t key, uint32_t idx) {
          if (select_equals_kth(key, idx, sh)) put(key, idx);
        });
      }
    }
  };
  uint32_t kk = 0;
  bool done = false;
#if MOL_FINAL_PREFIX
  if (row >= FINAL_PREFIX_MIN && row / 16 >= 2 * (int64_t)k && 24 * k <= SEG_CAP) {  // about 16 k entries reach the bound
    // a long row (single-level form): the k-th best key of its first sixteenth bounds the row's k-th best from below;
    // one pass over the row collects what reaches the bound into LDS and the selection runs there (as in k_seg_topk)
    auto each_prefix = [&](auto f) {
      block_for_each<4>(sc, row / 16, [&](int64_t i, float v) {
        const int32_t id = ci ? ci[i] : (int32_t)i;
        if (id >= 0) f(f32_to_key(v), (uint32_t)id);
      });
    };
    const uint32_t kp = block_select_kth<false>(each_prefix, (uint32_t)k, sh);
    const uint32_t bound = (kp == (uint32_t)k) ? sh.kth_key : 0u;
    __syncthreads();
    if (tid == 0) s_cnt = 0;
    __syncthreads();
    each([&](uint32_t key, uint32_t idx) {
      if (key >= bound) {
        const uint32_t slot = atomicAdd(&s_cnt, 1u);
        if (slot < SEG_CAP) s_buf[slot] = make_uint2(key, idx);
      }
    });
    __syncthreads();
    const uint32_t cnt = s_cnt;
    if (cnt <= SEG_CAP) {
      auto each_buf = [&](auto f) {
        for (uint32_t e = tid; e < cnt; e += SELECT_THREADS) {
          const uint2 v = s_buf[e];
          f(v.x, v.y);
        }
      };
      kk = block_select_kth<true>(each_buf, (uint32_t)k, sh);
      take(each_buf, kk);
      done = true;
    }
    __syncthreads();
  }
#endif
  if (!done) {
    kk = block_select_kth<true>(each, (uint32_t)k, sh);  // how many real results: min(k, valid candidates)
    take(each, kk);
  }
  __syncthreads();
  // bitonic sort of the first nsort slots (a power of two covering k; key desc, idx asc); one element per thread
  for (int size = 2; size <= nsort; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      const int i = tid, j = tid ^ stride;
      if (j > i && j < nsort) {
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

// slices per query of the two-level form (1 = single level)
#ifndef MOL_TOPK_SLICE
#define MOL_TOPK_SLICE 6144  // entries of a row one level-1 workgroup reduces (16 slices of a 1e5-candidate row)
#endif
#ifndef MOL_TOPK_MAXG
#define MOL_TOPK_MAXG 32
#endif
// A level-1 workgroup pays a fixed price per radix pass (histogram, scans, barriers), so large batches take fewer,
// longer slices: at most about 8192 level-1 workgroups per call, never fewer than 8 slices per query.
static int topk_slices(int B, int64_t Kp, int k) {
  int64_t G = Kp / MOL_TOPK_SLICE;
  if (G > MOL_TOPK_MAXG) G = MOL_TOPK_MAXG;
  int64_t by_batch = 4096 / (B > 0 ? B : 1);
  if (by_batch < 4) by_batch = 4;
  if (G > by_batch) G = by_batch;
  // a row of up to four slices is done faster by one workgroup (prefix bound + one collecting pass: 33 against 45 us at
  // K' = 16384, B = 128); a row of 1e5 is not (90 against 56 us at B = 32)
  if (G < 4 || G * (int64_t)k * 2 > Kp) G = 1;
  return (int)G;
}

size_t final_topk_workspace_bytes(int B, int64_t Kp, int k) {
  const int G = topk_slices(B, Kp, k);
  return G > 1 ? 2 * align_up((size_t)B * G * k * 4, 256) : 0;
}

mol_status_t launch_final_topk(const float *scores, const int32_t *cand_idx, const int32_t *cand_count, int B, int64_t Kp,
                               int k, int32_t *out_idx, float *out_score, char *ws, hipStream_t st) {
  if (k > TOPK_MAX) return mol_fail(MOL_EUNSUPPORTED, "k=%d exceeds the supported maximum %d", k, TOPK_MAX);
  ProfScope ps(MOL_PROF_FINAL_TOPK, st);
  int nsort = 64;
  while (nsort < k) nsort <<= 1;
  const int G = topk_slices(B, Kp, k);
  if (G > 1) {
    float *st_score = reinterpret_cast<float *>(ws);
    int32_t *st_idx = reinterpret_cast<int32_t *>(ws + align_up((size_t)B * G * k * 4, 256));
    hipLaunchKernelGGL(k_seg_topk, dim3(G, B), dim3(SELECT_THREADS), 0, st, scores, cand_idx, cand_count, Kp, k, st_score,
                       st_idx);
    HIP_TRY(hipGetLastError());
    scores = st_score;
    cand_idx = st_idx;
    cand_count = nullptr;
    Kp = (int64_t)G * k;
  }
  hipLaunchKernelGGL(k_final_topk, dim3(B), dim3(SELECT_THREADS), 0, st, scores, cand_idx, cand_count, Kp, k, nsort, out_idx,
                     out_score);
  HIP_TRY(hipGetLastError());
  return MOL_OK;
}
