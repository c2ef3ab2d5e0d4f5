// Multi-workgroup radix selection under the total order (key descending, index ascending).
//
// The lists handled here (sampled stage-1 scores, stage-1 survivors) hold 1e5..1e6
// entries per query: too much for one workgroup to walk several times at the latency the path needs, so every pass is
// a grid of (slices x queries) workgroups.  Three histogram passes over fixed digits of the 32-bit key
// (bits 31..21, 20..10, 9..0) find the exact K-th key; an emit pass writes everything above it, and the few items tied
// at the K-th key are parked in a small buffer from which a finishing workgroup takes the lowest indices.
// Where the caller knows a narrow key window that holds the K-th element (stage 1 does, from its sample), the
// histogram is one pass over 2048 equal slices of that window, made by whoever produces the elements, and the members
// of the slice that holds the K-th element are parked and ranked by the finishing workgroup.
// No per-query state is carried between the kernels except the three histograms: every workgroup re-derives the
// digits found so far from them (a 2048-bin scan, microseconds), which saves a launch per pass.
#pragma once
#include "common.hpp"

#define MSEL_THREADS 256
#define MSEL_BINS 2048
#define MSEL_PASSES 3
#define MSEL_TIE_CAP 2048

__device__ __forceinline__ int msel_lo(int p) { return p == 0 ? 21 : (p == 1 ? 10 : 0); }
__device__ __forceinline__ int msel_bins(int p) { return p == 2 ? 1024 : 2048; }

struct MselShared {
  uint32_t hist[MSEL_BINS];
  uint32_t part[MSEL_THREADS];
  uint32_t res[4];
};

// What the three histograms say about the K-th element of one query.
struct MselCut {
  uint32_t total;   // number of elements in the list
  uint32_t K;       // effective rank: min(requested, total)
  uint32_t prefix;  // key bits fixed by the passes resolved so far
  uint32_t krem;    // rank inside the set that matches prefix
  uint32_t cnt;     // size of the digit bucket chosen by the last resolved pass
};

// Workgroup-cooperative: the digit of pass-histogram g (nb bins) that holds rank krem (1-based from the largest digit).
// Returns through sh.res: {digit, rank inside the digit, bucket size, total}.  Requires 1 <= krem <= total for a
// meaningful digit; total is always right.
__device__ inline void msel_find(const uint32_t *g, int nb, uint32_t krem, MselShared &sh) {
  const int t = threadIdx.x;
  const int per = nb / MSEL_THREADS;
  const int top = nb - 1 - t * per;  // this thread covers digits top, top-1, ..., top-per+1
  uint32_t s = 0;
  for (int j = 0; j < per; ++j) s += g[top - j];
  if (t == 0) {
    sh.res[0] = 0;
    sh.res[1] = 0;
    sh.res[2] = 0;
  }
  // inclusive prefix over threads (thread 0 holds the largest digits): inside each wavefront with lane shuffles, then
  // the wavefront totals through LDS
  uint32_t incl_w = s;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t up = (uint32_t)__shfl_up((int)incl_w, o);
    if ((t & 63) >= o) incl_w += up;
  }
  if ((t & 63) == 63) sh.part[t >> 6] = incl_w;
  __syncthreads();
  uint32_t before = 0;
  for (int w = 0; w < (t >> 6); ++w) before += sh.part[w];
  const uint32_t incl = incl_w + before;
  uint32_t above = incl - s;
  if (t == MSEL_THREADS - 1) sh.res[3] = incl;
  if (above < krem && krem <= incl) {
    int d = top;
    uint32_t c = g[d];
    while (above + c < krem) {
      above += c;
      c = g[--d];
    }
    sh.res[0] = (uint32_t)d;
    sh.res[1] = krem - above;
    sh.res[2] = c;
  }
  __syncthreads();
}

// Re-derives the cut after `resolved` passes (0..3) from the per-pass histograms of query b.
// hist layout: [MSEL_PASSES][B][MSEL_BINS].
__device__ inline MselCut msel_cut(const uint32_t *hist, int B, int b, uint32_t K_req, int resolved, MselShared &sh) {
  MselCut c;
  c.total = 0;
  c.K = 0;
  c.prefix = 0;
  c.krem = 0;
  c.cnt = 0;
  for (int p = 0; p < resolved; ++p) {
    const uint32_t *g = hist + ((size_t)p * B + b) * MSEL_BINS;
    if (p == 0) {
      msel_find(g, msel_bins(0), 0xffffffffu, sh);  // only the total is used
      c.total = sh.res[3];
      c.K = K_req < c.total ? K_req : c.total;
      c.krem = c.K;
      __syncthreads();
      if (c.K == 0) return c;
    }
    msel_find(g, msel_bins(p), c.krem, sh);
    c.prefix |= sh.res[0] << msel_lo(p);
    c.krem = sh.res[1];
    c.cnt = sh.res[2];
    __syncthreads();
  }
  return c;
}

// Histogram pass p over the elements `each` hands out (each(f) calls f(key, idx) for this workgroup's slice).
// The caller provides the prefix fixed by the earlier passes.  Flushes non-empty bins to the global histogram.
template <class Each>
__device__ inline void msel_hist_pass(Each each, int p, uint32_t prefix, uint32_t *ghist, MselShared &sh) {
  const int nb = msel_bins(p);
  for (int i = threadIdx.x; i < nb; i += MSEL_THREADS) sh.hist[i] = 0;
  __syncthreads();
  const int lo = msel_lo(p);
  const int hi_shift = lo + (p == 2 ? 10 : 11);
  const uint32_t mask = (uint32_t)nb - 1u;
  each([&](uint32_t key, uint32_t) {
    const bool match = (p == 0) || ((key >> hi_shift) == (prefix >> hi_shift));
    if (match) atomicAdd(&sh.hist[(key >> lo) & mask], 1u);
  });
  __syncthreads();
  for (int i = threadIdx.x; i < nb; i += MSEL_THREADS) {
    const uint32_t v = sh.hist[i];
    if (v) atomicAdd(&ghist[i], v);
  }
}

// Appends (key, idx) to an output list with one atomic per wavefront.  `take` may differ per lane; all 64 lanes
// of the wavefront must call.
__device__ __forceinline__ uint32_t msel_wave_slot(bool take, uint32_t *counter) {
  const uint64_t m = __ballot(take);
  if (m == 0) return 0;
  const int lane = threadIdx.x & 63;
  const int leader = __ffsll((unsigned long long)m) - 1;
  uint32_t base = 0;
  if (lane == leader) base = atomicAdd(counter, (uint32_t)__popcll(m));
  base = __shfl(base, leader);
  return base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
}

// Walks slice `blk` of `nblk` of p[0..n) with U loads in flight per thread.  f(i, value, valid) is called the same
// number of times by every thread of the workgroup (valid = false past the end), so f may use wavefront collectives.
template <int U, class T, class F>
__device__ __forceinline__ void msel_slice_for_each(const T *p, int64_t n, int blk, int nblk, F f) {
  const int64_t step = (int64_t)U * MSEL_THREADS;
  int64_t chunk = (n + nblk - 1) / nblk;
  chunk = (chunk + step - 1) / step * step;
  const int64_t lo = (int64_t)blk * chunk;
  int64_t hi = lo + chunk;
  if (hi > n) hi = n;
  for (int64_t base = lo; base < hi; base += step) {
    T v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = base + (int64_t)u * MSEL_THREADS + threadIdx.x;
      if (i < hi) v[u] = p[i];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = base + (int64_t)u * MSEL_THREADS + threadIdx.x;
      f(i, v[u], i < hi);
    }
  }
}

// Finishing helper: of the nt entries (key, idx) parked in `parked`, the `need` first ones under the order (key
// descending, idx ascending) are handed to `put(slot, key, idx)`, every slot 0 .. need-1 once, in no particular order.
// One workgroup of MSEL_THREADS; nt <= MSEL_TIE_CAP; need <= nt.  `scratch` is LDS for MSEL_TIE_CAP entries.
// Few entries are ranked against each other; many (integer-valued scores put hundreds of equal keys into one slice)
// go through an 8-bit radix selection in LDS, four digits of the key and, where the cut falls inside a run of equal keys,
// four of the index.
template <class Put>
__device__ inline void msel_take_best(const uint2 *parked, uint32_t nt, uint32_t need, uint2 *scratch, MselShared &sh,
                                      Put put) {
  for (uint32_t i = threadIdx.x; i < nt; i += MSEL_THREADS) scratch[i] = parked[i];
  __syncthreads();
  if (nt <= MSEL_THREADS) {
    for (uint32_t i = threadIdx.x; i < nt; i += MSEL_THREADS) {
      const uint2 me = scratch[i];
      uint32_t rank = 0;
      for (uint32_t j = 0; j < nt; ++j) {
        const uint2 o = scratch[j];
        const bool before = o.x > me.x || (o.x == me.x && (o.y < me.y || (o.y == me.y && j < i)));
        rank += before ? 1u : 0u;
      }
      if (rank < need) put(rank, me.x, me.y);
    }
    __syncthreads();
    return;
  }
  uint32_t kth_key = 0, idx_limit = 0xffffffffu, prefix = 0, krem = need;
  bool on_idx = false;
  for (int pass = 0; pass < 8; ++pass) {
    const int shift = 24 - 8 * (pass & 3);
    for (int i = threadIdx.x; i < 256; i += MSEL_THREADS) sh.hist[i] = 0;
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < nt; i += MSEL_THREADS) {
      const uint2 e = scratch[i];
      const uint32_t v = on_idx ? ~e.y : e.x;
      bool match = !on_idx || e.x == kth_key;
      if (shift < 24) match = match && (v >> (shift + 8)) == (prefix >> (shift + 8));
      if (match) atomicAdd(&sh.hist[(v >> shift) & 255u], 1u);
    }
    __syncthreads();
    msel_find(sh.hist, 256, krem, sh);
    prefix |= sh.res[0] << shift;
    const uint32_t in_digit = sh.res[2];
    krem = sh.res[1];
    __syncthreads();
    if (pass == 3) {
      kth_key = prefix;
      if (krem == in_digit) break;  // every entry with the key at the cut is taken
      on_idx = true;
      prefix = 0;
    }
    if (pass == 7) idx_limit = ~prefix;
  }
  if (threadIdx.x == 0) sh.res[0] = 0;
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < nt; i += MSEL_THREADS) {
    const uint2 e = scratch[i];
    if (e.x > kth_key || (e.x == kth_key && e.y <= idx_limit)) {
      const uint32_t slot = atomicAdd(&sh.res[0], 1u);
      if (slot < need) put(slot, e.x, e.y);
    }
  }
  __syncthreads();
}

__global__ void k_zero_u32(uint32_t *p, size_t n);
#define MCNT_STRIDE 64  // uint32 per query in the counter block: [0] emitted, [1] ties parked
