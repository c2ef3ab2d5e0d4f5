// Block-wide radix selection under the total order (key descending, index ascending).
// One workgroup of SELECT_THREADS threads works on one list; the list stays in global memory (L2 resident)
// and is re-read once per radix pass.  Used for: the sampled threshold of stage 1, the reduction of the
// stage-1 survivors to K' candidates (Section 4.1.2), and the final top-k of stage 2 (Algorithm 1, last line).
#pragma once
#include "common.hpp"

#define SELECT_THREADS 1024
#define SELECT_BITS 11
#define SELECT_BINS (1 << SELECT_BITS)

struct SelectShared {
  alignas(16) uint32_t hist[SELECT_BINS];
  uint32_t chunk[64];
  uint32_t red_min[SELECT_THREADS / WAVE];
  uint32_t red_max[SELECT_THREADS / WAVE];
  uint32_t red_cnt[SELECT_THREADS / WAVE];
  uint32_t count;      // number of elements of the list
  uint32_t prefix;     // bits decided so far
  uint32_t krem;       // rank still to resolve inside the matching set
  uint32_t kmin, kmax;
  uint32_t kth_key;    // result: key of the K-th element
  uint32_t idx_limit;  // result: ties with key == kth_key are accepted while idx <= idx_limit
  uint32_t ties, out_count;
};

// Walks p[0..n) with the whole block, U independent loads in flight per thread: f(i, p[i]).
template <int U, class T, class F>
__device__ __forceinline__ void block_for_each(const T *p, int64_t n, F f) {
  for (int64_t base = threadIdx.x; base < n; base += (int64_t)U * SELECT_THREADS) {
    T v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = base + (int64_t)u * SELECT_THREADS;
      if (i < n) v[u] = p[i];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = base + (int64_t)u * SELECT_THREADS;
      if (i < n) f(i, v[u]);
    }
  }
}

// The list is given as a callable `each(f)` that calls f(key, idx) for every element this thread owns (the block's
// threads together cover the list exactly once; the same partition on every call is not required).
//
// One radix pass.  ON_IDX = false: digit of the key, among elements agreeing with sh.prefix above bit `hi`.
// ON_IDX = true: digit of ~idx among the elements whose key equals sh.kth_key.
// Two forms of the search for the digit that holds the wanted rank.  select_pass_narrow leaves it to the first
// wavefront (the other fifteen wait at the barrier and cost nothing): right where the device is full of such
// workgroups and instruction issue is what counts (level 1 of the final top-k at B = 1024).  select_pass gives every
// thread two bins: a third of the latency, sixteen times the instructions: right where one workgroup per query is all
// there is (thresholds, level 2 of the top-k).
template <bool ON_IDX, class Each>
__device__ void select_pass_narrow(Each each, int lo, int hi, SelectShared &sh) {
  const int tid = threadIdx.x;
  for (int i = tid; i < SELECT_BINS; i += SELECT_THREADS) sh.hist[i] = 0;
  __syncthreads();
  const uint32_t prefix = sh.prefix;
  const uint32_t kth_key = sh.kth_key;
  const int w = hi - lo + 1;
  const uint32_t dmask = (1u << w) - 1u;
  each([&](uint32_t key, uint32_t idx) {
    uint32_t k = key;
    bool valid = true;
    if (ON_IDX) {
      valid = key == kth_key;
      k = ~idx;  // ascending index == descending ~index
    }
    const bool match = (hi >= 31) ? true : ((k >> (hi + 1)) == (prefix >> (hi + 1)));
    if (valid && match) atomicAdd(&sh.hist[(k >> lo) & dmask], 1u);
  });
  __syncthreads();
  // locate the digit that holds rank krem counting from the largest digit: the first wavefront alone, with lane scans
  // (chunk t covers `per` consecutive digits from the top; then the lanes take one digit each of the chunk that holds it)
  const int nb = 1 << w;
  const int per = (nb + 63) / 64;  // digits per chunk (<= 32)
  if (tid < 64) {
    const uint32_t krem = sh.krem;
    uint32_t s = 0;
    const int top = nb - 1 - tid * per;
    for (int j = 0; j < per; ++j) {
      const int d = top - j;
      if (d >= 0) s += sh.hist[d];
    }
    uint32_t incl = s;  // inclusive sum over chunks 0..tid
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t up = (uint32_t)__shfl_up((int)incl, o);
      if (tid >= o) incl += up;
    }
    // first chunk whose inclusive sum reaches krem (the last chunk if none does: krem never exceeds the total)
    const uint64_t reach = __ballot(incl >= krem);
    const int c = reach ? __ffsll((unsigned long long)reach) - 1 : 63;
    const uint32_t before = (uint32_t)__shfl((int)(incl - s), c);  // elements in the chunks above chunk c
    // inside chunk c: lane j takes digit dtop - j
    const int dtop = nb - 1 - c * per;
    const int d_mine = dtop - tid;
    const uint32_t h = (tid < per && d_mine >= 0) ? sh.hist[d_mine] : 0u;
    uint32_t hin = h;
#pragma unroll
    for (int o = 1; o < 32; o <<= 1) {
      const uint32_t up = (uint32_t)__shfl_up((int)hin, o);
      if (tid >= o) hin += up;
    }
    const uint64_t hit = __ballot(tid < per && d_mine >= 0 && before + hin >= krem);
    int j = hit ? __ffsll((unsigned long long)hit) - 1 : (dtop < per ? dtop : per - 1);  // fall back to the chunk's last digit
    const uint32_t above = before + (uint32_t)__shfl((int)(hin - h), j);
    if (tid == 0) {
      const int d = dtop - j;
      sh.krem = krem - above;  // rank inside digit d
      sh.prefix = prefix | ((uint32_t)d << lo);
      sh.ties = sh.hist[d];
    }
  }
  __syncthreads();
}

// sh.hist must be all zero on entry and is all zero again on return.
template <bool ON_IDX, class Each>
__device__ void select_pass(Each each, int lo, int hi, SelectShared &sh) {
  static_assert(SELECT_BINS == 2 * SELECT_THREADS, "the digit search gives every thread two bins");
  const int tid = threadIdx.x;
  const uint32_t prefix = sh.prefix;
  const uint32_t kth_key = sh.kth_key;
  const uint32_t krem = sh.krem;
  const int w = hi - lo + 1;
  const uint32_t dmask = (1u << w) - 1u;
  each([&](uint32_t key, uint32_t idx) {
    uint32_t k = key;
    bool valid = true;
    if (ON_IDX) {
      valid = key == kth_key;
      k = ~idx;  // ascending index == descending ~index
    }
    const bool match = (hi >= 31) ? true : ((k >> (hi + 1)) == (prefix >> (hi + 1)));
    if (valid && match) atomicAdd(&sh.hist[(k >> lo) & dmask], 1u);
  });
  __syncthreads();
  // locate the digit that holds rank krem counting from the largest digit: thread t owns digits top-2t and top-2t-1
  // (read as one aligned pair and cleared for the next pass); inclusive sums run over the lanes of a wavefront, then
  // over the wavefronts through sh.chunk
  const int nb = 1 << w;
  const int p2 = SELECT_BINS / 2 - 1 - tid;  // pair index: bins 2*p2 (lower digit) and 2*p2+1 (higher digit)
  const uint2 pr = reinterpret_cast<uint2 *>(sh.hist)[p2];
  reinterpret_cast<uint2 *>(sh.hist)[p2] = make_uint2(0u, 0u);
  // digits at or above nb are never filled; thread t sees them as zero, so counting from the top of the table is the
  // same as counting from digit nb-1
  const uint32_t h_hi = pr.y, h_lo = pr.x;
  const uint32_t s = h_hi + h_lo;
  uint32_t incl = s;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t up = (uint32_t)__shfl_up((int)incl, o);
    if ((tid & 63) >= o) incl += up;
  }
  if ((tid & 63) == 63) sh.chunk[tid >> 6] = incl;
  __syncthreads();
  uint32_t before = 0;
  for (int i = 0; i < (tid >> 6); ++i) before += sh.chunk[i];
  incl += before;
  const uint32_t above = incl - s;  // elements in digits larger than this thread's pair
  if (above < krem && krem <= incl) {  // exactly one thread (1 <= krem <= number of matching elements)
    const bool in_hi = krem <= above + h_hi;
    const int d = 2 * p2 + (in_hi ? 1 : 0);
    sh.krem = krem - above - (in_hi ? 0u : h_hi);
    sh.prefix = prefix | ((uint32_t)d << lo);
    sh.ties = in_hi ? h_hi : h_lo;
  }
  (void)nb;
  __syncthreads();
}

// Finds the K-th element of the list, K clamped to the number of elements (returned; sh.count holds that number).
// On return sh.kth_key / sh.idx_limit describe the accepted set { key > kth_key } U { key == kth_key and
// idx <= idx_limit }, which has exactly the returned number of members; 0 is returned for an empty list or K = 0 and
// nothing may then be accepted.
// WITH_TIES = false skips the index stage (idx_limit = all ones): used when only the key value matters.
template <bool WITH_TIES, bool WIDE = true, class Each>
__device__ uint32_t block_select_kth(Each each, uint32_t K, SelectShared &sh) {
  const int tid = threadIdx.x;
  // 1. size of the list and range of the keys: bits above the highest differing bit are common and need no pass
  uint32_t mn = 0xffffffffu, mx = 0u, n_mine = 0;
  each([&](uint32_t key, uint32_t) {
    mn = min(mn, key);
    mx = max(mx, key);
    ++n_mine;
  });
  for (int o = 32; o > 0; o >>= 1) {
    mn = min(mn, (uint32_t)__shfl_xor((int)mn, o));
    mx = max(mx, (uint32_t)__shfl_xor((int)mx, o));
    n_mine += (uint32_t)__shfl_xor((int)n_mine, o);
  }
  if ((tid & 63) == 0) {
    sh.red_min[tid >> 6] = mn;
    sh.red_max[tid >> 6] = mx;
    sh.red_cnt[tid >> 6] = n_mine;
  }
  for (int i = tid; i < SELECT_BINS; i += SELECT_THREADS) sh.hist[i] = 0;  // the passes keep it zero between them
  __syncthreads();
  if (tid == 0) {
    for (int i = 1; i < SELECT_THREADS / WAVE; ++i) {
      mn = min(mn, sh.red_min[i]);
      mx = max(mx, sh.red_max[i]);
      n_mine += sh.red_cnt[i];
    }
    sh.count = n_mine;
    K = K < n_mine ? K : n_mine;
    sh.kmin = mn;
    sh.kmax = mx;
    sh.krem = K;
    uint32_t diff = mn ^ mx;
    // common high bits stay in prefix
    int hb = diff ? 31 - __clz(diff) : -1;
    sh.prefix = (hb >= 31) ? 0u : (hb < 0 ? mx : (mx >> (hb + 1)) << (hb + 1));
    sh.kth_key = 0;
    sh.idx_limit = 0xffffffffu;
    sh.ties = 0;
  }
  __syncthreads();
  K = sh.krem;  // the clamped rank, in every thread
  if (K == 0) return 0;
  {
    uint32_t diff = sh.kmin ^ sh.kmax;
    int hi = diff ? 31 - __clz(diff) : -1;
    while (hi >= 0) {
      int lo = hi - (SELECT_BITS - 1);
      if (lo < 0) lo = 0;
      if constexpr (WIDE) select_pass<false>(each, lo, hi, sh);
      else select_pass_narrow<false>(each, lo, hi, sh);
      hi = lo - 1;
    }
  }
  if (tid == 0) sh.kth_key = sh.prefix;
  __syncthreads();
  if (!WITH_TIES) return K;
  // 2. ties at the K-th key: keep the krem smallest indices among them
  //    (when the keys were all equal no pass ran and `ties` is not known: always resolve by index then)
  const bool all_equal = (sh.kmin == sh.kmax);
  if (!all_equal && sh.krem == sh.ties) return K;  // every tie is accepted
  __syncthreads();
  if (tid == 0) sh.prefix = 0;
  __syncthreads();
  for (int hi = 31; hi >= 0;) {
    int lo = hi - (SELECT_BITS - 1);
    if (lo < 0) lo = 0;
    if constexpr (WIDE) select_pass<true>(each, lo, hi, sh);
    else select_pass_narrow<true>(each, lo, hi, sh);
    hi = lo - 1;
  }
  if (tid == 0) sh.idx_limit = ~sh.prefix;
  __syncthreads();
  return K;
}

// What block_select_kth accepts, in two classes: entries that come before the K-th element in the total order, and
// entries equal to it in key and index.  A list may name an item more than once (a caller's candidate row), and then
// more entries may equal the K-th than there is room for: whoever collects the K results takes the first class whole
// (fewer than K entries when the second is not empty) and fills up from the second.
__device__ __forceinline__ bool select_before_kth(uint32_t key, uint32_t idx, const SelectShared &sh) {
  return key > sh.kth_key || (key == sh.kth_key && idx < sh.idx_limit);
}
__device__ __forceinline__ bool select_equals_kth(uint32_t key, uint32_t idx, const SelectShared &sh) {
  return key == sh.kth_key && idx == sh.idx_limit;
}
