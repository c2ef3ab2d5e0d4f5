// Stage 1, h-indexer (Section 4.1, Algorithm 2): sampled threshold, streaming corpus scan fused with the
// strict threshold filter, and the reduction of the survivors to K' candidates.
//
// The scan is a skinny GEMM (32*NQG queries x N items x d1) that is bound by reading the item table once
// (Section 4.1.1: arithmetic intensity ~ 2B/byteW).  Each wavefront owns tiles of 32 consecutive rows:
// it loads them straight into the matrix-core operand layout (lane = row, 16 bytes of the row per load), keeps
// the query fragments in registers for the whole kernel, accumulates in fp32 on MFMA and compares the 32x32
// score tile against the per-query thresholds in registers.  Only survivors are written (index + score key),
// so no N-length score vector ever reaches HBM.
//
// Survivor lists.  In the 32x32 score tile a lane always holds scores of ONE query (column = lane % 32), so every
// (wavefront, lane) pair appends the survivors it finds to a list of its own and counts them in a register: no
// atomics in the scan.  A query therefore owns L = 2 * (number of wavefronts) short lists; which wavefront gets a tile
// is fixed by the tile number, so each list is a deterministic set whatever the timing.  The lists one wavefront
// writes are adjacent in memory ([list][query][slot]).
#include <math.h>
#include <stdlib.h>

#include <atomic>

#include "common.hpp"
#include "msel.hpp"
#include "select.hpp"

// Tuning constants of the corpus scan (measured on MI355X at N = 1e8, B = 32).
#ifndef MOL_SCAN_DEPTH
#define MOL_SCAN_DEPTH 2     // tiles in flight per wavefront (register ring)
#endif
#ifndef MOL_SCAN_TILE_RUN
#define MOL_SCAN_TILE_RUN 4  // consecutive 32-row tiles a wavefront reads before it strides by the whole grid
#endif
#ifndef MOL_SCAN_PER_CU
#define MOL_SCAN_PER_CU 2    // resident workgroups per compute unit (bf16 / fp32 table)
#endif
#ifndef MOL_SCAN_PER_CU_I8
#define MOL_SCAN_PER_CU_I8 4 // int8 table (half the bytes per tile): more wavefronts, one tile in flight each
#endif
#ifndef MOL_SCAN_DEPTH_I8
#define MOL_SCAN_DEPTH_I8 1
#endif
#ifndef MOL_SCAN_DEPTH_Q4
#define MOL_SCAN_DEPTH_Q4 2  // tiles in flight per wavefront of the filtering scan with four query groups (queries in LDS)
#endif
#ifndef MOL_SCAN_WAVES_Q4
#define MOL_SCAN_WAVES_Q4 3  // ... and its wavefronts per SIMD
#endif

namespace {

// Survivor records a lane stages in LDS before it writes them out (per query group); the rings of a workgroup take
// 4 wavefronts * 64 lanes * NQG * entries * 8 bytes.
constexpr uint32_t scan_ring_entries(int nqg) { return nqg == 4 ? 4u : 16u; }
// The filtering scan with four query groups keeps the queries in LDS instead of 64 registers (every wavefront of a
// workgroup uses the same ones) and runs three wavefronts per SIMD: its 64 threshold compares per lane and tile are
// dependent compare / branch pairs, and a third wavefront hides more of them than the registers were worth.
constexpr bool scan_queries_in_lds(int epi, int nqg) { return epi == 0 /* EPI_FILTER */ && nqg == 4; }
// The corpus scan with one query group (the 32-query batch of the 100M-item workload) reads the table with streaming
// (non-temporal) loads, which only pay when every load instruction takes whole 128-byte lines: 7.1 instead of 6.3 TB/s
// for a bare read of 12.8 GB, but 3.3 instead of 2.05 ms for the scan when each line is shared by four instructions, as
// the operand layout (lane = row) has it.  So a wavefront loads a tile as it lies in memory (lane l: bytes 16 l .. 16 l + 15
// of each KB) and turns it into the operand layout through LDS.
#ifndef MOL_SCAN_STAGED
#define MOL_SCAN_STAGED 1
#endif
constexpr bool scan_staged(int epi, int nqg, bool gather) {
  return MOL_SCAN_STAGED && epi == 0 /* EPI_FILTER */ && nqg == 1 && !gather;
}
constexpr int scan_row_bytes(int dt) { return dt == MOL_F32 ? 256 : (dt == MOL_BF16 ? 128 : 64); }
constexpr int scan_chunks(int dt) { return dt == MOL_F32 ? 8 : (dt == MOL_BF16 ? 4 : 2); }

enum { EPI_FILTER = 0, EPI_KEYS = 1, EPI_HIST_KEY = 2, EPI_HIST_IDX = 3, EPI_FILTER_EXACT = 4 };

// Exact redo of a query whose sampled threshold missed (too few survivors, or a survivor list overflowed): a radix
// select over recomputed scores.  Four scans histogram the 8-bit digits of the score key (most significant first)
// and give the exact K'-th key; if only some of the items tied at that key may be taken, four more scans do the same
// on the item index among the ties (lowest indices win).  A last scan then keeps exactly the K' items
// {key > tkey} U {key == tkey, idx <= idx_limit} and writes them straight to the output (one counter per query hands
// out the slots: the K' items may sit in consecutive rows, e.g. a run of duplicates, so per-wavefront lists of bounded
// size cannot hold them).  Every kernel of the chain returns at once when no query is flagged, the normal case.
struct ExactState {
  uint32_t active;     // 0 not redone, 1 key passes, 2 index passes, 3 threshold known
  uint32_t prefix;     // digits found so far (of the key, then of ~idx)
  uint32_t krem;       // rank still to resolve
  uint32_t tkey;       // exact K'-th key
  uint32_t idx_limit;  // ties at tkey are taken while idx <= idx_limit
  uint32_t emitted;    // output slots handed out by the last scan
  uint32_t pad[2];
};
#define EXACT_BINS 256

struct ScanArgs {
  const char *X;         // item table, row-major, ROWB bytes per row
  int64_t n_rows;        // rows to score (N, or lambda for the gathered sample)
  const int32_t *rows;   // GATHER: row numbers into X
  int64_t x_rows;        // GATHER: number of rows of X (row numbers are clamped into range)
  const char *Q;         // queries, row-major, same dtype / width as X
  int B;                 // total number of queries
  int qbase;             // first query handled by this launch
  const float *thr;      // FILTER: per-query threshold (strict >)
  uint32_t *cnt;         // FILTER*: [B][L] survivors found per list (may exceed cap: overflow)
  uint2 *surv;           // FILTER*: [L][B][cap] (key, idx): the lists one wavefront writes are adjacent in memory
  int64_t L;             // lists per query = 2 * wavefronts of the launch
  int64_t cap;           // capacity of one list
  uint32_t *skeys;       // KEYS: [B][skeys_stride] score keys
  int64_t skeys_stride;
  ExactState *state;        // exact redo: per-query state
  int32_t *out_idx;         // FILTER_EXACT: [B][Kp] candidates, written directly
  float *out_score;         // FILTER_EXACT: [B][Kp] or NULL
  int32_t *out_count;       // FILTER_EXACT: [B]
  uint32_t *flags;          // FILTER_EXACT: [B] per-query status (1 = being redone -> 0 done / 3 failed)
  int Kp;
  uint32_t *gate_rw;        // exact redo: the two gate words and, at [2], the workgroup ticket of the redo scans
  int stage;                // exact redo: step to run when a histogram scan has finished (1..8)
  uint32_t idx_prefix;      // exact redo: digits of ~idx that are the same for every item (N <= 2^24: the top one is 0xff), not scanned for
  uint32_t *hist;           // exact redo: [B][EXACT_BINS] digit histogram
  const uint32_t *gate;     // exact redo: the kernel returns at once when *gate == 0
  int shift;                // exact redo: bit position of the digit
  int paper;                // FILTER_EXACT: Algorithm 2 as written -- of the K' best only those above the sampled threshold are kept
};

// Key window of one query, known from the sample before the corpus scan: the K'-th best score of the corpus lies in
// (t_key, u_key] unless the sample misleads (then the query is redone exactly).  One pass over the survivors counts
// them per slice of the window (2048 equal slices), which is enough to cut the K' best out of them: the members of the
// slice that holds the K'-th are ranked by a finishing workgroup.  (Counting in the scan itself, one global atomic
// per survivor, cost 120 us at N = 1e8: the atomics sit in the same in-order queue as the prefetched tiles.)
// Stored as uint2 {t_key, u_key} (the two ends are found by different workgroups); make_window() adds the shift:
// slice of a key = (key - t_key) >> shift, keys above u_key are not counted.
__device__ __forceinline__ uint32_t win_slice(uint32_t key, const uint4 w) {
  const uint32_t s = (key > w.x ? key - w.x : 0u) >> w.z;
  return s < (uint32_t)MSEL_BINS ? s : (uint32_t)MSEL_BINS - 1u;
}
__device__ __forceinline__ uint4 make_window(const uint2 tu) {
  const uint32_t t_key = tu.x, u_key = tu.y < tu.x ? tu.x : tu.y;
  const uint32_t w = u_key - t_key;
  const int bits = w ? 32 - __clz(w) : 0;
  return make_uint4(t_key, u_key, bits > 11 ? (uint32_t)(bits - 11) : 0u, 0u);
}
// upper end of the window when the sample is too small to bracket the K'-th score from above: as far above the largest
// sampled key as that key lies above the threshold
__device__ __forceinline__ uint32_t window_top_from_max(uint32_t t_key, uint32_t max_key) {
  if (max_key < t_key) max_key = t_key;
  const uint64_t u = (uint64_t)max_key + (uint64_t)(max_key - t_key) + 1024u;
  return u > 0xffffffffull ? 0xffffffffu : (uint32_t)u;
}

// One step of the exact redo, run for query b by the 256 threads of the last workgroup of a histogram scan to finish:
//   stage 1..4 : digit of the key found from the histogram of the scan just done; after the fourth the K'-th key is
//                known and either every tie is taken or the index passes start (gate[1] = 1).
//   stage 5..8 : the same on ~idx among the ties; after the fourth the index limit is known.
// The histogram row is read past the L1 cache (other workgroups added to it with device-scope atomics) and zeroed for
// the next scan.
__device__ inline void exact_step(int stage, uint32_t idx_prefix, ExactState *st, uint32_t *hb, uint32_t *gate, uint32_t *suf) {
  const int t = threadIdx.x;
  __syncthreads();  // suf and *st may still be in use by the previous query's step
  const uint32_t want = stage <= 4 ? 1u : 2u;
  const uint32_t active = st->active;
  const uint32_t mine = __hip_atomic_load(&hb[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  hb[t] = 0;  // ready for the next scan
  if (active != want) return;
  // inclusive suffix sums: suf[t] = sum of bins >= t
  suf[t] = mine;
  __syncthreads();
  for (int o = 1; o < EXACT_BINS; o <<= 1) {
    const uint32_t add = (t + o < EXACT_BINS) ? suf[t + o] : 0u;
    __syncthreads();
    suf[t] += add;
    __syncthreads();
  }
  const uint32_t krem = st->krem, prefix = st->prefix;
  const uint32_t above = suf[t] - mine;  // elements in larger digits
  __syncthreads();
  if (above < krem && krem <= above + mine) {  // exactly one thread
    const int shift = 24 - 8 * ((stage - 1) & 3);
    const uint32_t np = prefix | ((uint32_t)t << shift);
    const uint32_t nk = krem - above;
    if (stage == 4) {
      st->tkey = np;
      if (nk == mine) {  // all items tied at the K'-th key fit
        st->active = 3;
        st->idx_limit = 0xffffffffu;
      } else {
        st->active = 2;
        st->prefix = idx_prefix;
        st->krem = nk;
        gate[1] = 1;
      }
    } else if (stage == 8) {
      st->idx_limit = ~np;
      st->active = 3;
    } else {
      st->prefix = np;
      st->krem = nk;
    }
  }
}

// True in every thread of the last workgroup of the grid to get here (all writes of the others are then visible);
// the counter is left at zero for the next launch.
__device__ inline bool last_workgroup(uint32_t *ticket) {
  __shared__ uint32_t s_last;
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t t = atomicAdd(ticket, 1u);
    s_last = (t == gridDim.x - 1) ? 1u : 0u;
    if (s_last) *ticket = 0;
  }
  __syncthreads();
  return s_last != 0;
}

// DT = MOL_BF16: bf16 rows of 64 (128 B), 4 x 16-byte chunks per lane, one 32x32x16 MFMA per chunk.
// DT = MOL_F32 : fp32 rows of 64 (256 B), 8 x 16-byte chunks per lane, four 32x32x2 MFMAs per chunk.
// DT = MOL_INT8: int8 rows of 64 (64 B), 2 x 16-byte chunks per lane, one 32x32x32 integer MFMA per chunk; the int32
//                sums (|s| <= 64*127*127 < 2^24) are converted to fp32 exactly, so everything after the contraction
//                -- threshold compare, keys, selection -- is the same code and the same total order (Section 4.1.1:
//                the integer scores go to the selection as they are, no scale is applied).
// Lane (r = lane%32, h = lane/32) takes chunks 2*ci + h of row r; the query operand uses the same chunk
// numbering, so the contraction pairs equal positions whatever order the hardware walks them in.
#ifndef MOL_SCAN_MIN_WAVES
#define MOL_SCAN_MIN_WAVES 2  // keeps the 4-query-group variants at two wavefronts per SIMD (they need 260 registers otherwise)
#endif
template <int DT, int NQG, int EPI, bool GATHER, int DEPTH>
__global__ __launch_bounds__(256, scan_queries_in_lds(EPI, NQG) ? MOL_SCAN_WAVES_Q4 : MOL_SCAN_MIN_WAVES) void k_stage1_scan(ScanArgs a) {
  constexpr int NCH = DT == MOL_F32 ? 8 : (DT == MOL_BF16 ? 4 : 2);
  constexpr int ROWB = DT == MOL_F32 ? 256 : (DT == MOL_BF16 ? 128 : 64);
  constexpr bool REDO = EPI >= EPI_HIST_KEY;
  constexpr bool HIST = EPI == EPI_HIST_KEY || EPI == EPI_HIST_IDX;
  constexpr bool LISTS = EPI == EPI_FILTER;
  const int lane = threadIdx.x & 63;
  const int r = lane & 31, h = lane >> 5;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  const int64_t ntiles = (a.n_rows + 31) >> 5;
  extern __shared__ uint32_t lds_hist[];  // HIST: [32*NQG][EXACT_BINS];  FILTER: survivor rings, see below
  // FILTER: a lane stages its survivors in a private LDS ring of RING entries and copies the ring to its list in HBM
  // when it is full, so that the lists are written in whole 64/128-byte pieces.  (Appending each 8-byte record straight
  // to HBM cost a quarter of the scan's time: 4.6 M scattered partial-line writes at N = 1e8, K' = 1e5.)
  constexpr uint32_t RING = scan_ring_entries(NQG);
  constexpr bool QLDS = scan_queries_in_lds(EPI, NQG);
  constexpr bool STAGED = scan_staged(EPI, NQG, GATHER);
  constexpr int CPRW = ROWB / 16;      // 16-byte pieces per row
  constexpr int RPI = 64 / CPRW;       // rows one load instruction of a wavefront covers when it reads memory as it lies
  constexpr int STG_ROW = ROWB + 16;   // LDS row pitch of the staged tile (the padding keeps the transposed reads apart)
  if constexpr (REDO) {
    if (*a.gate == 0) return;
  }
  if constexpr (HIST) {
    for (int i = threadIdx.x; i < 32 * NQG * EXACT_BINS; i += 256) lds_hist[i] = 0;
    __syncthreads();
  }

  uint4 q[QLDS ? 1 : NQG][QLDS ? 1 : NCH];
  // QLDS: [NQG][NCH][64 lanes] behind the survivor rings
  uint4 *q_lds = reinterpret_cast<uint4 *>(reinterpret_cast<char *>(lds_hist) + (size_t)4 * 64 * NQG * RING * 8);
  // STAGED: one tile per wavefront, [32 rows][STG_ROW bytes], behind the rings
  char *stg = reinterpret_cast<char *>(lds_hist) + (size_t)4 * 64 * NQG * RING * 8 + (size_t)(threadIdx.x >> 6) * 32 * STG_ROW;
  float thr[NQG];
  int32_t thr_i[NQG];  // DT = MOL_INT8, FILTER only
  uint32_t st_active[NQG], st_prefix[NQG], st_tkey[NQG], st_ilim[NQG];
  uint32_t cnt[NQG];
  uint2 *lst[NQG];
  const uint32_t cap32 = (uint32_t)a.cap;
  uint2 *ring[NQG];
#pragma unroll
  for (int g = 0; g < NQG; ++g) {
    const int b = a.qbase + 32 * g + r;
    ring[g] = reinterpret_cast<uint2 *>(lds_hist) + ((size_t)((threadIdx.x >> 6) * NQG + g) * 64 + lane) * RING;
#pragma unroll
    for (int ci = 0; ci < NCH; ++ci) {
      const uint4 qv = (b < a.B) ? ld16(a.Q + (size_t)b * ROWB + (2 * ci + h) * 16) : make_uint4(0, 0, 0, 0);
      if constexpr (QLDS) {
        if (threadIdx.x < 64) q_lds[(g * NCH + ci) * 64 + lane] = qv;  // the same for every wavefront: the first one stores
      } else {
        q[g][ci] = qv;
      }
    }
    thr[g] = (EPI == EPI_FILTER && b < a.B) ? a.thr[b] : INFINITY;
    if constexpr (EPI == EPI_FILTER_EXACT) thr[g] = (a.paper && b < a.B) ? a.thr[b] : -INFINITY;
    // an int8 table: the filter compares the integer sums themselves (s > t  <=>  s > floor(t) for an integer s), which
    // saves the 16 conversions per tile and query group of a scan that is bound by instruction issue, not by memory
    if constexpr (DT == MOL_INT8 && EPI == EPI_FILTER) {
      const float t = floorf(thr[g]);
      thr_i[g] = t >= 2147483648.f ? 0x7fffffff : (t < -2147483648.f ? (int32_t)0x80000000 : (int32_t)t);
    }
    st_active[g] = 0;
    cnt[g] = 0;
    lst[g] = nullptr;
    if constexpr (LISTS) {
      if (b < a.B) lst[g] = a.surv + ((size_t)(wave * 2 + h) * a.B + b) * a.cap;
    }
    if constexpr (REDO) {
      if (b < a.B) {
        const ExactState s = a.state[b];
        st_active[g] = s.active;
        st_prefix[g] = s.prefix;
        st_tkey[g] = s.tkey;
        st_ilim[g] = s.idx_limit;
      }
    }
  }

  if constexpr (QLDS) __syncthreads();  // the queries are in LDS
  auto qop = [&](int g, int ci) -> uint4 {
    if constexpr (QLDS) return q_lds[(g * NCH + ci) * 64 + lane];
    else return q[g][ci];
  };

  auto load_tile = [&](uint4(&dst)[NCH], int64_t tile) {
    if constexpr (STAGED) {
#pragma unroll
      for (int ci = 0; ci < NCH; ++ci) {
        int64_t row = tile * 32 + ci * RPI + lane / CPRW;
        if (row >= a.n_rows) row = a.n_rows - 1;
        dst[ci] = ld16_stream(a.X + (size_t)row * ROWB + (lane % CPRW) * 16);
      }
      return;
    }
    int64_t row = tile * 32 + r;
    if (row >= a.n_rows) row = a.n_rows - 1;
    if (GATHER) {
      row = a.rows[row];
      row = row < 0 ? 0 : (row >= a.x_rows ? a.x_rows - 1 : row);
    }
    const char *p = a.X + (size_t)row * ROWB + h * 16;
#pragma unroll
    for (int ci = 0; ci < NCH; ++ci) dst[ci] = ld16(p + ci * 32);
  };

  // copies the first n (even up to RING) staged records of query group g to the lane's list; cnt[g] already counts them
  auto flush_ring = [&](int g, uint32_t n) __attribute__((always_inline)) {
    if (lst[g] == nullptr || cnt[g] > cap32) return;  // a list that overflowed is redone anyway
    uint2 *dst = lst[g] + (cnt[g] - n);
    for (uint32_t e = 0; e + 2 <= n; e += 2)
      *reinterpret_cast<uint4 *>(dst + e) = *reinterpret_cast<const uint4 *>(ring[g] + e);
    if (n & 1u) dst[n - 1] = ring[g][n - 1];
  };

  uint4 buf[DEPTH][NCH];
  // A wavefront reads TILE_RUN consecutive tiles (4 KB each at bf16), then jumps by the whole grid: the grid as a whole sweeps the
  // table front to back while each wavefront's loads stay within a DRAM page for a few steps.
  constexpr int64_t TILE_RUN = MOL_SCAN_TILE_RUN;
  const int64_t n_it = (ntiles + nwaves * TILE_RUN - 1) / (nwaves * TILE_RUN) * TILE_RUN;  // tiles per wavefront
  auto tile_of = [&](int64_t it) -> int64_t { return ((it / TILE_RUN) * nwaves + wave) * TILE_RUN + it % TILE_RUN; };
#pragma unroll
  for (int i = 0; i < DEPTH; ++i)
    if (i < n_it && tile_of(i) < ntiles) load_tile(buf[i], tile_of(i));

  // one tile out of ring slot tb (iteration `it` of this wavefront); false when the wavefront has no more tiles
  auto do_tile = [&](uint4(&tb)[NCH], int64_t it) __attribute__((always_inline)) -> bool {
    {
      if (it >= n_it) return false;
      const int64_t tile = tile_of(it);
      if (tile >= ntiles) return false;  // tile_of grows with its argument: nothing valid follows
      f32x16 acc[NQG];
      i32x16 iacc[NQG];  // DT = MOL_INT8 only
#pragma unroll
      for (int g = 0; g < NQG; ++g)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          acc[g][j] = 0.f;
          iacc[g][j] = 0;
        }
      uint4 op[STAGED ? NCH : 1];  // STAGED: the tile in operand layout (lane = row), read back from LDS
      if constexpr (STAGED) {
#pragma unroll
        for (int ci = 0; ci < NCH; ++ci)
          *reinterpret_cast<uint4 *>(stg + (ci * RPI + lane / CPRW) * STG_ROW + (lane % CPRW) * 16) = tb[ci];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int ci = 0; ci < NCH; ++ci) op[ci] = *reinterpret_cast<const uint4 *>(stg + r * STG_ROW + (2 * ci + h) * 16);
        // the ring slot is free as soon as it is in LDS: the next tile's loads start before this tile's arithmetic
        if (it + DEPTH < n_it) {
          const int64_t tnext = tile_of(it + DEPTH);
          if (tnext < ntiles) load_tile(tb, tnext);
        }
      }
      auto rowop = [&](int ci) -> uint4 {
        if constexpr (STAGED) return op[ci];
        else return tb[ci];
      };
#pragma unroll
      for (int ci = 0; ci < NCH; ++ci) {
#pragma unroll
        for (int g = 0; g < NQG; ++g) {
          if constexpr (DT == MOL_INT8) {
            iacc[g] = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_i32x4(rowop(ci)), as_i32x4(qop(g, ci)), iacc[g], 0, 0, 0);
          } else if constexpr (DT == MOL_F32) {
            const uint4 aa = rowop(ci);
            const float av[4] = {__uint_as_float(aa.x), __uint_as_float(aa.y), __uint_as_float(aa.z), __uint_as_float(aa.w)};
            const uint4 qq = qop(g, ci);
            const float qv[4] = {__uint_as_float(qq.x), __uint_as_float(qq.y), __uint_as_float(qq.z), __uint_as_float(qq.w)};
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[e], qv[e], acc[g], 0, 0, 0);
          } else {
            acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(rowop(ci)), as_bf16x8(qop(g, ci)), acc[g], 0,
                                                             0, 0);
          }
        }
      }
      if (!STAGED && it + DEPTH < n_it) {
        const int64_t tnext = tile_of(it + DEPTH);
        if (tnext < ntiles) load_tile(tb, tnext);
      }
      mfma_settle();
      constexpr bool INT_FILTER = DT == MOL_INT8 && EPI == EPI_FILTER;
      if constexpr (DT == MOL_INT8 && !INT_FILTER) {
#pragma unroll
        for (int g = 0; g < NQG; ++g)
#pragma unroll
          for (int j = 0; j < 16; ++j) acc[g][j] = (float)iacc[g][j];
      }

      // acc[g][j]: item row 8*(j/4) + 4*h + j%4 of the tile, query qbase + 32*g + r
      const int64_t row0 = tile * 32 + 4 * h;
#pragma unroll
      for (int g = 0; g < NQG; ++g) {
        const int b = a.qbase + 32 * g + r;
        if constexpr (EPI == EPI_FILTER) {
          // about 1.5 of the 1024 scores of a tile pass: one compare per accumulator, and the (rare) append is a
          // branch the wavefront skips when no lane takes it
          auto append = [&](int j) __attribute__((always_inline)) {
            const float sc = INT_FILTER ? (float)iacc[g][j] : acc[g][j];  // |sum| < 2^24: exact
            ring[g][cnt[g] & (RING - 1)] = make_uint2(f32_to_key(sc), (uint32_t)(row0 + 8 * (j >> 2) + (j & 3)));
            ++cnt[g];
            if ((cnt[g] & (RING - 1)) == 0) flush_ring(g, RING);
          };
          auto passes = [&](int gg, int j) -> bool {
            if constexpr (INT_FILTER) return iacc[gg][j] > thr_i[gg];
            else return acc[gg][j] > thr[gg];
          };
          if (tile != ntiles - 1) {
            // the wavefront-wide test first: when no lane passes (all but ~2 % of the compares) the cost is the compare
            // and one scalar branch on its mask, with no save / restore of the execution mask
#pragma unroll
            for (int j = 0; j < 16; ++j)
              if (__builtin_amdgcn_ballot_w64(passes(g, j)) != 0) [[unlikely]] {
                if (passes(g, j)) append(j);
              }
          } else {
#pragma unroll
            for (int j = 0; j < 16; ++j)
              if (passes(g, j) && row0 + 8 * (j >> 2) + (j & 3) < a.n_rows) append(j);  // the last tile can be partial
          }
        } else if constexpr (EPI == EPI_FILTER_EXACT) {
          if (st_active[g] == 3u) {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
              const int64_t n = row0 + 8 * (j >> 2) + (j & 3);
              const uint32_t k = f32_to_key(acc[g][j]);
              if ((k > st_tkey[g] || (k == st_tkey[g] && (uint32_t)n <= st_ilim[g])) && n < a.n_rows &&
                  acc[g][j] > thr[g]) {
                const uint32_t slot = atomicAdd(&a.state[b].emitted, 1u);
                if (slot < (uint32_t)a.Kp) {  // at most K' items qualify; the check only guards the buffer
                  a.out_idx[(size_t)b * a.Kp + slot] = (int32_t)n;
                  if (a.out_score) a.out_score[(size_t)b * a.Kp + slot] = key_to_f32(k);
                }
              }
            }
          }
        } else if constexpr (HIST) {
          if (st_active[g] == (EPI == EPI_HIST_KEY ? 1u : 2u)) {
            uint32_t *hrow = lds_hist + (32 * g + r) * EXACT_BINS;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
              const int64_t n = row0 + 8 * (j >> 2) + (j & 3);
              const uint32_t key = f32_to_key(acc[g][j]);
              const uint32_t k = (EPI == EPI_HIST_KEY) ? key : ~(uint32_t)n;
              bool take = n < a.n_rows;
              if (EPI == EPI_HIST_IDX) take = take && key == st_tkey[g];
              if (a.shift < 24) take = take && (k >> (a.shift + 8)) == (st_prefix[g] >> (a.shift + 8));
              if (take) atomicAdd(&hrow[(k >> a.shift) & (EXACT_BINS - 1)], 1u);
            }
          }
        } else {
          if (b < a.B) {
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
              uint4 kv = make_uint4(f32_to_key(acc[g][4 * qd]), f32_to_key(acc[g][4 * qd + 1]),
                                    f32_to_key(acc[g][4 * qd + 2]), f32_to_key(acc[g][4 * qd + 3]));
              *reinterpret_cast<uint4 *>(a.skeys + (size_t)b * a.skeys_stride + row0 + 8 * qd) = kv;
            }
          }
        }
      }
    }
    return true;
  };
  static_assert(DEPTH >= 1 && DEPTH <= 6, "ring slots are walked by hand");
  for (int64_t it0 = 0; it0 < n_it; it0 += DEPTH) {
    if (!do_tile(buf[0], it0)) break;
    if constexpr (DEPTH > 1)
      if (!do_tile(buf[1], it0 + 1)) break;
    if constexpr (DEPTH > 2)
      if (!do_tile(buf[2], it0 + 2)) break;
    if constexpr (DEPTH > 3)
      if (!do_tile(buf[3], it0 + 3)) break;
    if constexpr (DEPTH > 4)
      if (!do_tile(buf[4], it0 + 4)) break;
    if constexpr (DEPTH > 5)
      if (!do_tile(buf[5], it0 + 5)) break;
  }
  if constexpr (LISTS) {
#pragma unroll
    for (int g = 0; g < NQG; ++g) {
      const int b = a.qbase + 32 * g + r;
      const uint32_t rest = cnt[g] & (RING - 1);
      if (rest) flush_ring(g, rest);
      if (b < a.B) a.cnt[(size_t)b * a.L + wave * 2 + h] = cnt[g];
    }
  }
  if constexpr (HIST) {
    __syncthreads();
    for (int i = threadIdx.x; i < 32 * NQG * EXACT_BINS; i += 256) {
      const uint32_t v = lds_hist[i];
      const int b = a.qbase + i / EXACT_BINS;
      if (v && b < a.B) atomicAdd(&a.hist[(size_t)b * EXACT_BINS + (i & (EXACT_BINS - 1))], v);
    }
    // the last workgroup to finish turns the histograms into the next digit of every query of this launch
    if (last_workgroup(a.gate_rw + 2)) {
      uint32_t *suf = lds_hist;  // the LDS histogram is flushed: reuse its first EXACT_BINS words
      for (int b = a.qbase; b < a.B && b < a.qbase + 32 * NQG; ++b)
        exact_step(a.stage, a.idx_prefix, a.state + b, a.hist + (size_t)b * EXACT_BINS, a.gate_rw, suf);
    }
  }
  if constexpr (EPI == EPI_FILTER_EXACT) {
    // the last workgroup closes the redo: a redone query holds exactly K' candidates (Algorithm 2 as written: those of
    // the K' best that lie above the sampled threshold, so possibly fewer; the unused slots are padded); anything else
    // (a threshold that was never resolved, a count that does not fit) is reported as cand_count = -1 with an empty row
    if (last_workgroup(a.gate_rw + 2)) {
      for (int b = a.qbase; b < a.B && b < a.qbase + 32 * NQG; ++b) {
        if (a.flags[b] == 0u) continue;  // not redone
        const uint32_t emitted = __hip_atomic_load(&a.state[b].emitted, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool ok = a.state[b].active == 3u && (a.paper ? emitted <= (uint32_t)a.Kp : emitted == (uint32_t)a.Kp);
        for (int i = (ok ? (int)emitted : 0) + threadIdx.x; i < a.Kp; i += 256) {
          a.out_idx[(size_t)b * a.Kp + i] = -1;
          if (a.out_score) a.out_score[(size_t)b * a.Kp + i] = -INFINITY;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
          a.out_count[b] = ok ? (int32_t)emitted : -1;
          a.flags[b] = ok ? 0u : 3u;
        }
      }
    }
  }
}

// i-th sampled row: floor(N * hi32(SplitMix64 output i) / 2^32), stream state = seed + (i+1) * golden gamma.
__device__ __forceinline__ int32_t sample_row(uint64_t seed, int64_t i, uint64_t N) {
  uint64_t z = seed + (uint64_t)(i + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z = z ^ (z >> 31);
  return (int32_t)(((z >> 32) * N) >> 32);
}
// The same launch clears `nz` words at `zero` (the histograms and counters of the two radix selections of the call).
__global__ void k_gen_sample(int32_t *out, int64_t lambda, uint64_t seed, uint64_t N, uint32_t *zero, size_t nz) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (size_t z = (size_t)i; z < nz; z += (size_t)gridDim.x * blockDim.x) zero[z] = 0u;
  if (i < lambda) out[i] = sample_row(seed, i, N);
}

// Per query: threshold = the rank-th largest sampled score (Algorithm 2, nthElement), by multi-workgroup radix
// selection over the B x lambda score keys.  k_thr_hist is launched once per digit pass; k_thr_finish writes the
// threshold and resets the flags and the redo gate.  The same sweeps find the rank_u-th largest key (the top of the
// query's key window) in a histogram set of its own: the first pass counts every key for both, the later ones count a
// key for whichever of the two prefixes it matches.
__global__ __launch_bounds__(MSEL_THREADS) void k_thr_hist(const uint32_t *skeys, int64_t stride, int64_t lambda,
                                                           uint32_t rank, uint32_t rank_u, uint32_t *mhist,
                                                           uint32_t *mhist_u, int B, int pass) {
  __shared__ MselShared sh;
  __shared__ uint32_t hist_u[MSEL_BINS];
  const int b = blockIdx.y, blk = blockIdx.x, G = gridDim.x;
  uint32_t prefix = 0, prefix_u = 0;
  if (pass > 0) {
    prefix = msel_cut(mhist, B, b, rank, pass, sh).prefix;
    if (rank_u) prefix_u = msel_cut(mhist_u, B, b, rank_u, pass, sh).prefix;
  }
  const uint32_t *keys = skeys + (size_t)b * stride;  // rows are 16-byte aligned (stride is a multiple of 32 keys)
  const int nb = msel_bins(pass);
  for (int i = threadIdx.x; i < nb; i += MSEL_THREADS) {
    sh.hist[i] = 0;
    hist_u[i] = 0;
  }
  __syncthreads();
  const int lo = msel_lo(pass);
  const int hi_shift = lo + (pass == 2 ? 10 : 11);
  const uint32_t mask = (uint32_t)nb - 1u;
  const bool both = rank_u != 0 && pass > 0;
  auto count = [&](uint32_t key) {
    const uint32_t d = (key >> lo) & mask;
    if (pass == 0 || (key >> hi_shift) == (prefix >> hi_shift)) atomicAdd(&sh.hist[d], 1u);
    if (both && (key >> hi_shift) == (prefix_u >> hi_shift)) atomicAdd(&hist_u[d], 1u);
  };
  const int64_t n4 = lambda >> 2;
  msel_slice_for_each<4>(reinterpret_cast<const uint4 *>(keys), n4, blk, G, [&](int64_t, uint4 v, bool valid) {
    if (valid) {
      count(v.x);
      count(v.y);
      count(v.z);
      count(v.w);
    }
  });
  if (blk == 0)
    for (int64_t i = 4 * n4 + threadIdx.x; i < lambda; i += MSEL_THREADS) count(keys[i]);
  __syncthreads();
  uint32_t *g = mhist + ((size_t)pass * B + b) * MSEL_BINS, *gu = mhist_u + ((size_t)pass * B + b) * MSEL_BINS;
  for (int i = threadIdx.x; i < nb; i += MSEL_THREADS) {
    const uint32_t v = sh.hist[i];
    if (v) atomicAdd(&g[i], v);
    const uint32_t vu = pass == 0 ? v : hist_u[i];
    if (rank_u && vu) atomicAdd(&gu[i], vu);
  }
}

// `passes` digit passes were made: 3 give the exact rank-th sampled key (Algorithm 2 as written); with 2 the threshold is
// the lower end of the 22-bit bucket holding it, at most 2^10 ulps below -- enough where the threshold only has to let
// at least K' items through (the exact top-K' of the survivors is taken afterwards) and one pass over the keys cheaper.
// The upper end of the query's key window is the rank_u-th sampled key (its bucket's upper end), rank_u < rank chosen
// by the host so that the K'-th best score of the corpus lies below it; rank_u = 0: no such rank exists in the sample.
__global__ __launch_bounds__(MSEL_THREADS) void k_thr_finish(const uint32_t *mhist, const uint32_t *mhist_u, int B,
                                                             uint32_t rank, uint32_t rank_u, int passes, float *thr,
                                                             uint2 *win, uint32_t *flags, uint32_t *gate) {
  __shared__ MselShared sh;
  const int b = blockIdx.x;
  const MselCut c = msel_cut(mhist, B, b, rank, passes, sh);
  // without a rank for the window top: the largest sampled key, as far as the first pass (which counts every key)
  // resolves it
  const MselCut cu = rank_u ? msel_cut(mhist_u, B, b, rank_u, passes, sh) : msel_cut(mhist, B, b, 1u, 1, sh);
  if (threadIdx.x == 0) {
    const uint32_t t_key = c.K ? c.prefix : f32_to_key(-INFINITY);
    uint32_t u_key = 0xffffffffu;
    if (cu.K) u_key = rank_u ? (cu.prefix | (passes < MSEL_PASSES ? 0x3ffu : 0u)) : window_top_from_max(t_key, cu.prefix | 0x1fffffu);
    thr[b] = key_to_f32(t_key);
    win[b] = make_uint2(t_key, u_key);
    flags[b] = 0;
    if (b == 0) gate[0] = gate[1] = gate[2] = 0;
  }
}

// The same for a set of keys that fits the LDS of one workgroup (THR_KEYS_CAP keys), exactly: threshold = the rank-th
// largest key, window top = the rank_u-th largest.  The keys of query b are either a dense row (dense + b * stride,
// n_dense of them) or the survivor lists of a filtering scan over the sampled rows (lists / cnt / L / lcap as the scan
// wrote them).  The second form serves large samples: a first, small part of the sample gives a bracket value
// `fallback` below which the rank-th key cannot lie, the scan over the whole sample keeps only the scores above the
// bracket, and this kernel picks the rank-th of those -- the B x lambda score matrix never exists.  Whatever the lists
// lost (more entries than a list or the LDS holds) only lowers the rank-th key of what is left, so the threshold errs
// to the side of more survivors; with fewer than `rank` entries the bracket itself is the threshold.
// Grid (B, 1 or 2): workgroup (b, 0) finds the threshold, (b, 1) the window top (win != NULL), side by side.
#define THR_KEYS_CAP 32768
__global__ __launch_bounds__(SELECT_THREADS) void k_thr_select(const uint32_t *dense, int64_t stride, int64_t n_dense,
                                                               const uint2 *lists, const uint32_t *cnt, int64_t L, int B,
                                                               uint32_t lcap, uint32_t kcap, uint32_t rank,
                                                               uint32_t rank_u, const float *fallback, float *thr,
                                                               uint2 *win, uint32_t *flags, uint32_t *gate) {
  extern __shared__ uint32_t s_keys[];  // kcap keys
  __shared__ SelectShared sh;
  __shared__ uint32_t s_n;
  const int b = blockIdx.x, tid = threadIdx.x;
  const bool top = blockIdx.y == 1;
  if (tid == 0) s_n = 0;
  __syncthreads();
  if (dense != nullptr) {
    const uint32_t *k = dense + (size_t)b * stride;
    for (int64_t i = tid; i < n_dense && i < kcap; i += SELECT_THREADS) s_keys[i] = k[i];
    if (tid == 0) s_n = (uint32_t)(n_dense < kcap ? n_dense : kcap);
  } else {
    // a thread takes U lists at a time and reads the first E entries of each in one go (a list of the sample scan
    // holds about one entry); places in s_keys come from a scan of the counts over the workgroup, not from atomics
    constexpr int U = 4, E = 4;
    uint32_t run = 0;  // keys placed so far, the same in every thread
    for (int64_t l0 = 0; l0 < L; l0 += (int64_t)U * SELECT_THREADS) {
      uint32_t c[U];
      uint2 v[U][E];
      uint32_t tc = 0;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t l = l0 + tid + (int64_t)u * SELECT_THREADS;
        c[u] = l < L ? cnt[(size_t)b * L + l] : 0u;
        if (c[u] > lcap) c[u] = lcap;
        tc += c[u];
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t l = l0 + tid + (int64_t)u * SELECT_THREADS;
#pragma unroll
        for (int e = 0; e < E; ++e)
          v[u][e] = (uint32_t)e < c[u] ? lists[((size_t)l * B + b) * lcap + e] : make_uint2(0u, 0u);
      }
      uint32_t incl = tc;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = (uint32_t)__shfl_up((int)incl, o);
        if ((tid & 63) >= o) incl += up;
      }
      if ((tid & 63) == 63) sh.chunk[tid >> 6] = incl;
      __syncthreads();
      uint32_t woff = 0, total = 0;
      for (int i = 0; i < SELECT_THREADS / 64; ++i) {
        const uint32_t t = sh.chunk[i];
        if (i < (tid >> 6)) woff += t;
        total += t;
      }
      uint32_t pos = run + woff + incl - tc;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t l = l0 + tid + (int64_t)u * SELECT_THREADS;
        for (uint32_t e = 0; e < c[u]; ++e, ++pos) {
          uint32_t key;
          if (e < (uint32_t)E) {
            key = v[u][0].x;
#pragma unroll
            for (int q = 1; q < E; ++q) key = e == (uint32_t)q ? v[u][q].x : key;
          } else {
            key = lists[((size_t)l * B + b) * lcap + e].x;
          }
          if (pos < kcap) s_keys[pos] = key;
        }
      }
      run += total;
      __syncthreads();  // sh.chunk is reused by the next round
    }
    if (tid == 0) s_n = run;
  }
  __syncthreads();
  const uint32_t n = s_n < kcap ? s_n : kcap;
  auto each = [&](auto f) {
    for (uint32_t i = tid; i < n; i += SELECT_THREADS) f(s_keys[i], 0u);
  };
  const uint32_t floor_key = fallback ? f32_to_key(fallback[b]) : f32_to_key(-INFINITY);
  if (!top) {
    uint32_t t_key = floor_key;
    if (n >= rank && rank >= 1) {  // the same in every thread
      block_select_kth<false>(each, rank, sh);
      t_key = sh.kth_key;
    }
    if (tid == 0) {
      thr[b] = key_to_f32(t_key);
      if (win) win[b].x = t_key;
      if (flags) flags[b] = 0;
      if (gate && b == 0) gate[0] = gate[1] = gate[2] = 0;
    }
  } else {
    uint32_t u_key = 0xffffffffu;
    if (rank_u >= 1 && n >= rank_u) {
      block_select_kth<false>(each, rank_u, sh);
      u_key = sh.kth_key;
    } else if (rank_u == 0) {
      // no sampled rank bounds the K'-th score from above: go as far above the largest sampled key as the (rank/2)-th
      // sampled key lies below it
      uint32_t mid = floor_key, mx = floor_key;
      if (n >= 1) {
        block_select_kth<false>(each, rank / 2 > 0 ? rank / 2 : 1u, sh);
        mid = sh.kth_key;
        mx = sh.kmax;
      }
      u_key = window_top_from_max(mid, mx);
    }
    if (tid == 0) win[b].y = u_key;
  }
}

// Bracket step of the large-sample threshold: workgroup b scores the first n0 sampled rows against query b with plain
// vector arithmetic (a few thousand dot products, too few to be worth a pass of the matrix-core scan and a second
// launch), keeps the keys in LDS and writes the rank0-th largest as thr0[b].  The value only has to lie below the
// rank-th score of the whole sample, so the summation order (not that of the scan) does not matter.
#define THR_BRACKET_ROWS 4096
template <int DT>
__global__ __launch_bounds__(SELECT_THREADS) void k_thr_bracket(const char *X, int64_t x_rows, const int32_t *rows,
                                                                int n0, const char *Q, uint32_t rank0, float *thr0) {
  constexpr int ROWB = DT == MOL_F32 ? 256 : (DT == MOL_BF16 ? 128 : 64);
  __shared__ SelectShared sh;
  __shared__ uint32_t s_keys[THR_BRACKET_ROWS];
  const int b = blockIdx.x, tid = threadIdx.x;
  // LG consecutive lanes share a row, 16 bytes each (one load instruction fetches 64 / LG whole rows); a lane keeps its
  // 16 bytes of the query decoded in registers
  constexpr int LG = ROWB / 16;
  constexpr int EL = DT == MOL_F32 ? 4 : (DT == MOL_BF16 ? 8 : 16);  // elements in 16 bytes
  const int part = tid % LG;
  auto decode = [](const uint4 v, float(&out)[EL]) {
    const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if constexpr (DT == MOL_F32) {
        out[e] = __uint_as_float(wv[e]);
      } else if constexpr (DT == MOL_BF16) {
        out[2 * e] = __uint_as_float(wv[e] << 16);
        out[2 * e + 1] = __uint_as_float(wv[e] & 0xffff0000u);
      } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) out[4 * e + t] = (float)(int8_t)((wv[e] >> (8 * t)) & 0xffu);
      }
    }
  };
  float qv[EL];
  decode(ld16(Q + (size_t)b * ROWB + 16 * part), qv);
  constexpr int RPI = SELECT_THREADS / LG;  // rows per step of the workgroup
  constexpr int UNR = 16;  // rows in flight per lane group
  for (int i0 = tid / LG; i0 < n0; i0 += UNR * RPI) {
    uint4 v[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int i = i0 + u * RPI < n0 ? i0 + u * RPI : i0;
      int64_t row = rows[i];
      row = row < 0 ? 0 : (row >= x_rows ? x_rows - 1 : row);
      v[u] = ld16(X + (size_t)row * ROWB + 16 * part);
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      float xv[EL];
      decode(v[u], xv);
      float acc = 0.f;
#pragma unroll
      for (int e = 0; e < EL; ++e) acc = fmaf(xv[e], qv[e], acc);
#pragma unroll
      for (int o = LG / 2; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
      const int i = i0 + u * RPI;
      if (part == 0 && i < n0) s_keys[i] = f32_to_key(acc);
    }
  }
  __syncthreads();
  auto each = [&](auto f) {
    for (int i = tid; i < n0; i += SELECT_THREADS) f(s_keys[i], 0u);
  };
  uint32_t key = f32_to_key(-INFINITY);
  if ((uint32_t)n0 >= rank0 && rank0 >= 1) {
    block_select_kth<false>(each, rank0, sh);
    key = sh.kth_key;
  }
  if (tid == 0) thr0[b] = key_to_f32(key);
}

__global__ void k_init_all_pass(float *thr, uint32_t *flags, uint32_t *gate, int B) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i == 0) gate[0] = gate[1] = gate[2] = 0;
  if (i < B) {
    thr[i] = -INFINITY;
    flags[i] = 0;
  }
}

// ---- survivors -> at most K' candidates (Section 4.1.2) ----------------------------------------------------------
// sstat[b] = {survivors of query b, 1 if its lists cannot give the answer}: a list overflowed, or (exact mode) fewer
// than K' survived, or the caller asked for the redo.  Such a query is left to the exact redo.  Workgroup-cooperative;
// every thread returns the value.
__device__ inline uint2 surv_status(const uint32_t *cnt, int64_t L, int64_t cap, int Kp, int mode, bool force, int b) {
  __shared__ uint32_t s_tot[MSEL_THREADS / 64], s_ovf[MSEL_THREADS / 64];
  uint32_t tot = 0, ovf = 0;
  for (int64_t i = threadIdx.x; i < L; i += MSEL_THREADS) {
    const uint32_t c = cnt[(size_t)b * L + i];
    tot += c;
    ovf |= ((int64_t)c > cap) ? 1u : 0u;
  }
  for (int o = 32; o > 0; o >>= 1) {
    tot += __shfl_xor((int)tot, o);
    ovf |= (uint32_t)__shfl_xor((int)ovf, o);
  }
  if ((threadIdx.x & 63) == 0) {
    s_tot[threadIdx.x >> 6] = tot;
    s_ovf[threadIdx.x >> 6] = ovf;
  }
  __syncthreads();
  tot = 0;
  ovf = 0;
  for (int i = 0; i < MSEL_THREADS / 64; ++i) {
    tot += s_tot[i];
    ovf |= s_ovf[i];
  }
  const bool bad = ovf || force || (mode == MOL_HINDEXER_EXACT && tot < (uint32_t)Kp);
  return make_uint2(tot, bad ? 1u : 0u);
}

// Walks lists [lo, hi) of query b.  A wavefront takes 32 lists at a time: the lanes fetch the counts with one load, then
// the lists are read sixteen at a time (independent loads in flight), LPL lanes across the entries of one list (32 where
// a list holds about 30 entries, N = 1e8 and 32 queries; 8 where it holds three or four, N = 1e7 and 128 queries).
// f(entry, valid) is called the same number of times by all 64 lanes of a wavefront (wavefront collectives are safe).
template <int LPL, class F>
__device__ __forceinline__ void for_each_survivor(const uint2 *surv, const uint32_t *cnt, int64_t L, int64_t cap, int B, int b,
                                                  int64_t lo, int64_t hi, int nwaves_in_block, F f) {
  static_assert(LPL == 32 || LPL == 16 || LPL == 8, "lanes per list");
  constexpr int LPW = 64 / LPL;  // lists one load instruction of a wavefront covers
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int which = lane / LPL, sub = lane % LPL;
  const uint32_t cap32 = (uint32_t)cap;
  constexpr int CHUNK = 32;        // lists a wavefront takes at a time (small, so that all wavefronts of a workgroup get lists)
  constexpr int UNR = 16 / LPW;    // load instructions in flight: 16 lists
  for (int64_t l0 = lo + (int64_t)wv * CHUNK; l0 < hi; l0 += (int64_t)nwaves_in_block * CHUNK) {
    uint32_t mine = 0;  // lane j (and j + 32) holds the count of list l0 + j
    if (l0 + (lane & 31) < hi) mine = cnt[(size_t)b * L + l0 + (lane & 31)];
    if (mine > cap32) mine = cap32;
    const int nl = (int)((hi - l0) < CHUNK ? (hi - l0) : CHUNK);
    const uint2 *base = surv + ((size_t)l0 * B + b) * cap;  // list l of query b starts at (l * B + b) * cap
    const size_t lstride = (size_t)B * cap;
    for (int i0 = 0; i0 < nl; i0 += LPW * UNR) {
      uint32_t n[UNR], nmax[UNR];
      uint2 v[UNR];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {  // lane group `which` of the wavefront reads list i0 + LPW * u + which
        const int li = i0 + LPW * u + which;
        const uint32_t from = (uint32_t)__shfl((int)mine, li & 31);  // by every lane: the lane read from must be active
        n[u] = (li < nl) ? from : 0u;
        uint32_t mx = n[u];  // the longest of the LPW lists: every lane makes that many rounds
#pragma unroll
        for (int o = LPL; o < 64; o <<= 1) {
          const uint32_t other = (uint32_t)__shfl_xor((int)mx, o);
          mx = other > mx ? other : mx;
        }
        nmax[u] = mx;
        v[u] = make_uint2(0u, 0u);
        if ((uint32_t)sub < n[u]) v[u] = base[(size_t)li * lstride + sub];
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        if (nmax[u]) f(v[u], (uint32_t)sub < n[u]);
        for (uint32_t e0 = LPL; e0 < nmax[u]; e0 += LPL) {  // lists longer than a lane group
          const uint32_t e = e0 + sub;
          const bool valid = e < n[u];
          uint2 w = make_uint2(0u, 0u);
          if (valid) w = base[(size_t)(i0 + LPW * u + which) * lstride + e];
          f(w, valid);
        }
      }
    }
  }
}

// Pass 0 also works out the query's status from the list counts (every workgroup for itself; the first one records it
// for the passes and kernels that follow).  With key windows (win != NULL) there is only pass 0, over the slices of the
// query's window instead of the first key digit.
template <int LPL>
__global__ __launch_bounds__(MSEL_THREADS) void k_surv_hist(const uint2 *surv, const uint32_t *cnt, int64_t L,
                                                            int64_t cap, uint2 *sstat, int Kp, uint32_t *mhist,
                                                            const uint2 *win, int B, int pass, int mode, bool force) {
  __shared__ MselShared sh;
  const int b = blockIdx.y, blk = blockIdx.x, G = gridDim.x;
  uint2 stt;
  if (pass == 0) {
    stt = surv_status(cnt, L, cap, Kp, mode, force, b);
    if (blk == 0 && threadIdx.x == 0) sstat[b] = stt;
  } else {
    stt = sstat[b];
  }
  if (stt.y || stt.x <= (uint32_t)Kp) return;
  const int64_t per = (L + G - 1) / G;
  const int64_t lo = blk * per, hi = lo + per < L ? lo + per : L;
  auto each = [&](auto f) {
    for_each_survivor<LPL>(surv, cnt, L, cap, B, b, lo, hi, MSEL_THREADS / 64, [&](uint2 e, bool valid) {
      if (valid) f(e.x, e.y);
    });
  };
  if (win != nullptr) {
    const uint4 w = make_window(win[b]);
    for (int i = threadIdx.x; i < MSEL_BINS; i += MSEL_THREADS) sh.hist[i] = 0;
    __syncthreads();
    each([&](uint32_t key, uint32_t) {
      if (key <= w.y) atomicAdd(&sh.hist[win_slice(key, w)], 1u);
    });
    __syncthreads();
    for (int i = threadIdx.x; i < MSEL_BINS; i += MSEL_THREADS) {
      const uint32_t v = sh.hist[i];
      if (v) atomicAdd(&mhist[(size_t)b * MSEL_BINS + i], v);
    }
    return;
  }
  uint32_t prefix = 0;
  if (pass > 0) prefix = msel_cut(mhist, B, b, (uint32_t)Kp, pass, sh).prefix;
  msel_hist_pass(each, pass, prefix, mhist + ((size_t)pass * B + b) * MSEL_BINS, sh);
}

// Where the K'-th best survivor of query b lies, worked out by every workgroup that needs it (256 threads).
//   kind 0: every survivor is taken;  kind 2: the lists cannot give the answer (exact redo);
//   kind 1: survivors of class > d are taken, of class d the `need` best of its `cbin` members (all of them when
//           need == cbin).  The class of a key is the key itself when three digit passes were made over the survivors
//           (win == NULL: d is the K'-th key), else its slice of the query's key window, keys above the window counting
//           as the highest class (the scan has counted the slices; those above are the rest of the total).
struct SurvCut {
  uint32_t kind, d, need, cbin;
  uint4 w;
  bool windowed;
  __device__ __forceinline__ uint32_t cls(uint32_t key) const {
    if (!windowed) return key;
    return key > w.y ? (uint32_t)MSEL_BINS : win_slice(key, w);
  }
};
__device__ inline SurvCut surv_cut(uint2 stt, int Kp, const uint32_t *mhist, const uint2 *win, int B, int b,
                                   MselShared &sh) {
  SurvCut c = {};
  c.windowed = win != nullptr;
  if (stt.y) {
    c.kind = 2;
    return c;
  }
  if (stt.x <= (uint32_t)Kp) return c;
  c.kind = 1;
  if (c.windowed) {
    c.w = make_window(win[b]);
    const uint32_t *g = mhist + (size_t)b * MSEL_BINS;
    msel_find(g, MSEL_BINS, 0xffffffffu, sh);  // only the total is used
    const uint32_t inwin = sh.res[3];
    __syncthreads();
    if (inwin > stt.x || stt.x - inwin >= (uint32_t)Kp) {  // the K'-th best lies above the window: the sample misled
      c.kind = 2;
      return c;
    }
    msel_find(g, MSEL_BINS, (uint32_t)Kp - (stt.x - inwin), sh);
    c.d = sh.res[0];
    c.need = sh.res[1];
    c.cbin = sh.res[2];
    __syncthreads();
  } else {
    const MselCut m = msel_cut(mhist, B, b, (uint32_t)Kp, MSEL_PASSES, sh);
    c.d = m.prefix;
    c.need = m.krem;
    c.cbin = m.cnt;
  }
  return c;
}

// Closes query b after the emit pass: ranks the parked members of the
// class at the cut, pads the row, writes cand_count, and sets up the exact redo when the lists cannot give the answer
// (or more members are parked than the buffer holds).
__device__ inline void surv_finish(const SurvCut &c, uint2 stt, int Kp, int b, const uint2 *tiebuf, uint2 *s_tie,
                                   MselShared &sh, uint32_t *flags, uint32_t *gate, ExactState *state, uint32_t *ehist,
                                   int32_t *cand_idx, float *cand_score, int32_t *cand_count) {
  const int tid = threadIdx.x;
  const bool redo = c.kind == 2 || (c.kind == 1 && c.need != c.cbin && c.cbin > MSEL_TIE_CAP);
  // state of the exact redo: a flagged query starts the key passes at rank K'
  if (tid == 0) {
    ExactState s = {};
    if (redo) {
      s.active = 1;
      s.krem = (uint32_t)Kp;
      s.idx_limit = 0xffffffffu;
    }
    state[b] = s;
  }
  for (int i = tid; i < EXACT_BINS; i += MSEL_THREADS) ehist[(size_t)b * EXACT_BINS + i] = 0;
  int32_t *oi = cand_idx + (size_t)b * Kp;
  float *os = cand_score ? cand_score + (size_t)b * Kp : nullptr;
  uint32_t nout = 0;
  if (redo) {
    if (tid == 0) {
      flags[b] = 1u;  // redone by the exact path
      gate[0] = 1u;
      cand_count[b] = -1;
    }
  } else if (c.kind == 0) {
    nout = stt.x;
    if (tid == 0) cand_count[b] = (int32_t)nout;
  } else {
    nout = (uint32_t)Kp;
    if (c.need != c.cbin) {  // only the `need` best of the cbin parked members of the class at the cut are taken
      const uint32_t base = (uint32_t)Kp - c.need;
      msel_take_best(tiebuf + (size_t)b * MSEL_TIE_CAP, c.cbin, c.need, s_tie, sh, [&](uint32_t rank, uint32_t key, uint32_t idx) {
        oi[base + rank] = (int32_t)idx;
        if (os) os[base + rank] = key_to_f32(key);
      });
    }
    if (tid == 0) cand_count[b] = Kp;
  }
  for (int64_t i = nout + tid; i < Kp; i += MSEL_THREADS) {
    oi[i] = -1;
    if (os) os[i] = -INFINITY;
  }
}

// win == NULL: sstat and the three digit histograms come from k_surv_hist.  Otherwise this kernel works the status out
// itself (every workgroup for itself; the first one records it for k_surv_finish) and mhist is the window histogram.
// (Closing the query in the last of its workgroups to finish, instead of a kernel of its own, was four times slower: the
// device-scope fence each workgroup needs before its ticket writes back the whole L2 of its XCD.)
template <int LPL>
__global__ __launch_bounds__(MSEL_THREADS) void k_surv_emit(const uint2 *surv, const uint32_t *cnt, int64_t L,
                                                            int64_t cap, uint2 *sstat, int Kp, const uint32_t *mhist,
                                                            const uint2 *win, int B, int mode, bool force,
                                                            uint32_t *mcnt, uint2 *tiebuf, int32_t *cand_idx,
                                                            float *cand_score) {
  __shared__ MselShared sh;
  const int b = blockIdx.y, blk = blockIdx.x, G = gridDim.x;
  uint2 stt;
  if (win != nullptr) {
    stt = surv_status(cnt, L, cap, Kp, mode, force, b);
    __syncthreads();
  } else {
    stt = sstat[b];
  }
  const SurvCut c = surv_cut(stt, Kp, mhist, win, B, b, sh);
  if (win != nullptr && blk == 0 && threadIdx.x == 0) sstat[b] = make_uint2(stt.x, c.kind == 2 ? 1u : 0u);
  if (c.kind == 2) return;
  uint32_t *mc = mcnt + (size_t)b * MCNT_STRIDE;
  const bool take_all = c.kind == 0;
  const bool all_ties = c.need == c.cbin;
  int32_t *oi = cand_idx + (size_t)b * Kp;
  float *os = cand_score ? cand_score + (size_t)b * Kp : nullptr;
  const int64_t per = (L + G - 1) / G;
  const int64_t lo = blk * per, hi = lo + per < L ? lo + per : L;
  // Two walks over this workgroup's lists: the first counts what each wavefront will emit, one atomic reserves the
  // workgroup's output range, the second writes (a returning atomic per wavefront step would serialise on latency).
  __shared__ uint32_t wave_tot[MSEL_THREADS / 64];
  __shared__ uint32_t block_base;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  uint32_t mine = 0;
  for_each_survivor<LPL>(surv, cnt, L, cap, B, b, lo, hi, MSEL_THREADS / 64, [&](uint2 e, bool valid) {
    const uint32_t k = c.cls(e.x);
    const bool at = valid && !take_all && k == c.d;
    const bool take = valid && (take_all || k > c.d || (at && all_ties));
    mine += (uint32_t)__popcll(__ballot(take));
  });
  if (lane == 0) wave_tot[wv] = mine;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t tot = 0;
    for (int i = 0; i < MSEL_THREADS / 64; ++i) tot += wave_tot[i];
    block_base = tot ? atomicAdd(mc, tot) : 0u;
  }
  __syncthreads();
  uint32_t off = block_base;
  for (int i = 0; i < wv; ++i) off += wave_tot[i];
  for_each_survivor<LPL>(surv, cnt, L, cap, B, b, lo, hi, MSEL_THREADS / 64, [&](uint2 e, bool valid) {
    const uint32_t k = c.cls(e.x);
    const bool at = valid && !take_all && k == c.d;
    const bool take = valid && (take_all || k > c.d || (at && all_ties));
    const bool tie = at && !all_ties;
    const uint64_t m = __ballot(take);
    const uint32_t slot = off + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
    off += (uint32_t)__popcll(m);
    if (take && slot < (uint32_t)Kp) {
      oi[slot] = (int32_t)e.y;
      if (os) os[slot] = key_to_f32(e.x);
    }
    if (__ballot(tie)) {
      const uint32_t ts = msel_wave_slot(tie, mc + 1);
      if (tie && ts < MSEL_TIE_CAP) tiebuf[(size_t)b * MSEL_TIE_CAP + ts] = e;
    }
  });
}

__global__ __launch_bounds__(MSEL_THREADS) void k_surv_finish(const uint2 *sstat, int Kp, const uint32_t *mhist,
                                                              const uint2 *win, int B, const uint2 *tiebuf,
                                                              uint32_t *flags, uint32_t *gate, ExactState *state,
                                                              uint32_t *ehist, int32_t *cand_idx, float *cand_score,
                                                              int32_t *cand_count) {
  __shared__ MselShared sh;
  __shared__ uint2 s_tie[MSEL_TIE_CAP];
  const int b = blockIdx.x;
  const uint2 stt = sstat[b];
  const SurvCut c = surv_cut(stt, Kp, mhist, win, B, b, sh);
  surv_finish(c, stt, Kp, b, tiebuf, s_tie, sh, flags, gate, state, ehist, cand_idx, cand_score, cand_count);
}

// ---- launch helpers ----------------------------------------------------------------------------------------------
template <int DT, int EPI, bool GATHER>
void (*scan_kernel(int nqg))(ScanArgs) {
  constexpr int DEPTH = DT == MOL_INT8 ? MOL_SCAN_DEPTH_I8 : MOL_SCAN_DEPTH;
  constexpr int DEPTH4 = scan_queries_in_lds(EPI, 4) ? (DT == MOL_INT8 ? 1 : MOL_SCAN_DEPTH_Q4) : DEPTH;
  return nqg == 4 ? k_stage1_scan<DT, 4, EPI, GATHER, DEPTH4>
                  : (nqg == 2 ? k_stage1_scan<DT, 2, EPI, GATHER, DEPTH> : k_stage1_scan<DT, 1, EPI, GATHER, DEPTH>);
}

// Queries one scan launch serves (a wavefront keeps them all in registers): 128, or 64 for an fp32 table, whose operands
// are twice as wide and would not leave room for two wavefronts per SIMD.
constexpr int scan_query_span(int dt) { return dt == MOL_F32 ? 64 : 128; }

// dynamic LDS of one scan workgroup
size_t scan_lds_bytes(int epi, int nqg, int dt) {
  if (epi == EPI_HIST_KEY || epi == EPI_HIST_IDX) return (size_t)32 * nqg * EXACT_BINS * 4;
  if (epi == EPI_FILTER)
    return (size_t)4 * 64 * nqg * scan_ring_entries(nqg) * 8 +
           (scan_queries_in_lds(epi, nqg) ? (size_t)nqg * scan_chunks(dt) * 64 * 16 : 0) +
           // the staged tile of each wavefront (the gathering variant of the same shape does not use it)
           (scan_staged(epi, nqg, false) ? (size_t)4 * 32 * (scan_row_bytes(dt) + 16) : 0);
  return 0;
}

int device_cus() {
  static std::atomic<int> cus{0};  // one GPU per process: the first answer is kept
  int v = cus.load(std::memory_order_relaxed);
  if (!v) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
      v = 0;
    cus.store(v, std::memory_order_relaxed);
  }
  return v;
}

// Workgroups (of 4 wavefronts) a scan over `ntiles` tiles is launched with: resident blocks, at most one tile each.
// fixed_grid > 0 forces the grid (the survivor lists are laid out for a given number of wavefronts).
// Resident workgroups per compute unit of one scan variant: asked of the runtime once per process and variant (the
// answer, and the raised LDS limit that goes with it, do not change afterwards), so that a call makes no HIP queries.
template <int DT, int EPI, bool GATHER>
mol_status_t scan_occupancy(int nqg, int *per_sm_out) {
  static std::atomic<int> cached[5] = {};  // by nqg (1, 2, 4); 0 = not asked yet
  int v = cached[nqg].load(std::memory_order_acquire);
  if (v == 0) {
    auto kern = scan_kernel<DT, EPI, GATHER>(nqg);
    const size_t lds = scan_lds_bytes(EPI, nqg, DT);
    if (lds > 48 * 1024)
      HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&v, kern, 256, lds));
    if (v < 1) v = 1;
    cached[nqg].store(v, std::memory_order_release);
  }
  *per_sm_out = v;
  return MOL_OK;
}

template <int DT, int EPI, bool GATHER>
mol_status_t scan_grid(int nqg, int64_t ntiles, int64_t *grid_out) {
  int per_sm = 0;
  mol_status_t rc = scan_occupancy<DT, EPI, GATHER>(nqg, &per_sm);
  if (rc != MOL_OK) return rc;
  constexpr int PER_CU = DT == MOL_INT8 ? MOL_SCAN_PER_CU_I8 : MOL_SCAN_PER_CU;
  const int per_cu = (scan_queries_in_lds(EPI, nqg) && PER_CU < MOL_SCAN_WAVES_Q4) ? MOL_SCAN_WAVES_Q4 : PER_CU;
  if (per_sm > per_cu) per_sm = per_cu;
  const int cus = device_cus();
  if (cus <= 0) return mol_fail(MOL_EHIP, "cannot query the device");
  int64_t grid = (int64_t)cus * per_sm;
  const int64_t need = (ntiles + 4 * MOL_SCAN_TILE_RUN - 1) / (4 * MOL_SCAN_TILE_RUN);  // at least one run of tiles for each of the 4 wavefronts
  if (grid > need) grid = need;
  if (grid < 1) grid = 1;
  *grid_out = grid;
  return MOL_OK;
}

template <int DT, int EPI, bool GATHER>
mol_status_t launch_scan(const ScanArgs &a0, int B, int64_t fixed_grid, hipStream_t st) {
  const int64_t ntiles = (a0.n_rows + 31) / 32;
  const int span = scan_query_span(DT);
  for (int qb = 0; qb < B; qb += span) {
    ScanArgs a = a0;
    a.qbase = qb;
    const int rem = B - qb < span ? B - qb : span;
    const int nqg = rem > 64 ? 4 : (rem > 32 ? 2 : 1);
    auto kern = scan_kernel<DT, EPI, GATHER>(nqg);
    int64_t grid = 0;
    mol_status_t rc = scan_grid<DT, EPI, GATHER>(nqg, ntiles, &grid);
    if (rc != MOL_OK) return rc;
    if (fixed_grid > 0) grid = fixed_grid;
    const size_t lds = scan_lds_bytes(EPI, nqg, DT);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, a);
    HIP_TRY(hipGetLastError());
  }
  return MOL_OK;
}

// The grid of the list-writing scan of a call: the smallest over the query-group variants the call will launch, so
// that the list layout (L = 8 * grid lists per query) is the same for all of them.
// launch_scan / scan_grid for a run-time stage-1 dtype
template <int EPI, bool GATHER>
mol_status_t launch_scan_dt(int dt, const ScanArgs &a, int B, int64_t fixed_grid, hipStream_t st) {
  switch (dt) {
    case MOL_F32: return launch_scan<MOL_F32, EPI, GATHER>(a, B, fixed_grid, st);
    case MOL_BF16: return launch_scan<MOL_BF16, EPI, GATHER>(a, B, fixed_grid, st);
    case MOL_INT8: return launch_scan<MOL_INT8, EPI, GATHER>(a, B, fixed_grid, st);
  }
  return mol_fail(MOL_EINVAL, "unknown stage-1 dtype %d", dt);
}

mol_status_t list_scan_grid(int dt, int B, int64_t N, int64_t *grid_out) {
  const int64_t ntiles = (N + 31) / 32;
  int64_t best = -1;
  const int span = scan_query_span(dt);
  for (int qb = 0; qb < B; qb += span) {
    const int rem = B - qb < span ? B - qb : span;
    const int nqg = rem > 64 ? 4 : (rem > 32 ? 2 : 1);
    int64_t g = 0;
    mol_status_t rc = dt == MOL_F32 ? scan_grid<MOL_F32, EPI_FILTER, false>(nqg, ntiles, &g)
                                    : (dt == MOL_BF16 ? scan_grid<MOL_BF16, EPI_FILTER, false>(nqg, ntiles, &g)
                                                      : scan_grid<MOL_INT8, EPI_FILTER, false>(nqg, ntiles, &g));
    if (rc != MOL_OK) return rc;
    if (best < 0 || g < best) best = g;
  }
  *grid_out = best;
  return MOL_OK;
}

}  // namespace

__global__ void k_zero_u32(uint32_t *p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// ------------------------------------------------------------------------------------------------ host
mol_status_t hindexer_plan(const mol_corpus *c, int B, int Kp, int64_t lambda, int mode, HindexerPlan *p) {
  const int64_t N = c->N;
  p->sampling = (4 * (int64_t)Kp < N);
  if (lambda <= 0) lambda = hindexer_default_lambda(c, Kp);
  if (lambda > N) lambda = N;
  if (lambda < 1) lambda = 1;
  p->lambda = p->sampling ? lambda : 0;
  int64_t r_paper = ((int64_t)Kp * lambda) / N;
  if (r_paper < 1) r_paper = 1;
  int64_t rank = r_paper;
  if (mode == MOL_HINDEXER_EXACT) rank = r_paper + (int64_t)ceil(5.0 * sqrt((double)r_paper)) + 8;
  if (rank > lambda) rank = lambda;
  p->rank = rank;
  // the K'-th best score of the corpus sits near sample rank K' * lambda / N: the same five standard deviations on the
  // other side bound it from above
  p->rank_u = r_paper - (int64_t)ceil(5.0 * sqrt((double)r_paper)) - 8;
  if (p->rank_u < 1 || p->rank_u >= rank) p->rank_u = 0;

  mol_status_t rc = list_scan_grid(c->stage1_dtype, B, N, &p->grid);
  if (rc != MOL_OK) return rc;
  p->L = p->grid * 8;  // 4 wavefronts per workgroup, 2 lists (lane halves) per wavefront
  // rows one list can see: the tiles of its wavefront, 16 rows of each
  const int64_t ntiles = (N + 31) / 32;
  const int64_t run_tiles = p->grid * 4 * MOL_SCAN_TILE_RUN;  // tiles one sweep of the grid covers
  const int64_t list_rows = (ntiles + run_tiles - 1) / run_tiles * MOL_SCAN_TILE_RUN * 16;  // rows that can land in one list
  if (p->sampling) {
    const double expect = (double)N * (double)rank / (double)lambda;
    double tot = expect * (1.0 + 6.0 / sqrt((double)rank)) + 1024;
    if (tot < (double)Kp + 1024) tot = (double)Kp + 1024;
    const double per = tot / (double)p->L;
    int64_t cap = (int64_t)(per + 8.0 * sqrt(per) + 8.0);
    cap = (cap + 15) & ~(int64_t)15;  // whole rings: a full ring either fits a list or overflows it
    if (cap > list_rows) cap = list_rows;
    p->cap = cap;
  } else {
    p->cap = list_rows;
  }
  // how the threshold is taken (see HindexerPlan::thr_path)
  p->thr_path = 0;
  p->lambda0 = 0;
  p->rank0 = 0;
  if (p->sampling) {
    p->thr_path = 3;
    if (p->lambda <= THR_KEYS_CAP) {
      p->thr_path = 1;
    } else if (mode == MOL_HINDEXER_EXACT) {
      const int64_t lam0 = THR_BRACKET_ROWS;
      const double m = (double)lam0 * (double)rank / (double)p->lambda;  // expected rows of the first part above the rank-th score
      int64_t rank0 = (int64_t)ceil(m + 6.0 * sqrt(m) + 4.0);
      if (rank0 > lam0) rank0 = lam0;
      const double kept = (double)p->lambda * (double)rank0 / (double)lam0;  // sampled scores expected above the bracket
      if (kept <= 8192.0 && kept <= 2.0 * (double)p->L) {
        p->thr_path = 2;
        p->lambda0 = lam0;
        p->rank0 = rank0;
      }
    }
  }
  const int64_t lam_pad = (p->lambda + 31) / 32 * 32;
  size_t off = 0;
  p->off_sample = off;
  off = align_up(off + (size_t)lam_pad * 4, 256);
  p->off_skeys = off;
  off = align_up(off + (size_t)B * (p->thr_path == 2 ? p->lambda0 : lam_pad) * 4, 256);
  p->off_thr = off;
  off = align_up(off + (size_t)B * 4, 256);
  p->off_thr0 = off;
  off = align_up(off + (size_t)B * 4, 256);
  p->off_win = off;
  off = align_up(off + (size_t)B * 16, 256);
  p->off_count = off;
  off = align_up(off + (size_t)B * p->L * 4, 256);
  p->off_flags = off;
  off = align_up(off + (size_t)B * 4, 256);
  p->off_sstat = off;
  off = align_up(off + (size_t)B * 8, 256);
  p->off_surv = off;
  off = align_up(off + (size_t)B * p->L * p->cap * 8, 256);
  p->off_mhist = off;  // three sets of radix-select histograms (sampled threshold, survivors, window top), then counters
  off = align_up(off + (size_t)3 * MSEL_PASSES * B * MSEL_BINS * 4, 256);
  p->off_mcnt = off;
  off = align_up(off + (size_t)B * MCNT_STRIDE * 4, 256);
  p->off_tie = off;
  off = align_up(off + (size_t)B * MSEL_TIE_CAP * 8, 256);
  p->off_hist = off;
  off = align_up(off + (size_t)B * EXACT_BINS * 4, 256);
  p->off_state = off;
  off = align_up(off + (size_t)B * sizeof(ExactState) + 256, 256);  // + the gate words and the ticket
  p->total = off;
  return MOL_OK;
}

mol_status_t hindexer_run(const mol_corpus *c, const void *q1, int B, int Kp, const int32_t *sample_idx,
                          uint64_t seed, int mode, const HindexerPlan &p, int32_t *cand_idx, float *cand_score,
                          int32_t *cand_count, char *ws, hipStream_t st) {
  const int dt = c->stage1_dtype;
  float *thr = reinterpret_cast<float *>(ws + p.off_thr);
  uint32_t *cnt = reinterpret_cast<uint32_t *>(ws + p.off_count);
  uint32_t *flags = reinterpret_cast<uint32_t *>(ws + p.off_flags);
  uint2 *sstat = reinterpret_cast<uint2 *>(ws + p.off_sstat);
  uint2 *surv = reinterpret_cast<uint2 *>(ws + p.off_surv);
  uint32_t *hist = reinterpret_cast<uint32_t *>(ws + p.off_hist);
  uint32_t *gate = reinterpret_cast<uint32_t *>(ws + p.off_state);
  ExactState *state = reinterpret_cast<ExactState *>(ws + p.off_state + 256);
  const bool force_redo = (mode & MOL_HINDEXER_FORCE_REDO) != 0;
  const bool defer_redo = (mode & MOL_HINDEXER_DEFER_REDO) != 0;
  mode &= ~(MOL_HINDEXER_FORCE_REDO | MOL_HINDEXER_DEFER_REDO);

  uint32_t *mhist = reinterpret_cast<uint32_t *>(ws + p.off_mhist);
  uint32_t *mhist2 = mhist + (size_t)MSEL_PASSES * B * MSEL_BINS;
  uint32_t *mhist_u = mhist2 + (size_t)MSEL_PASSES * B * MSEL_BINS;
  uint32_t *mcnt = reinterpret_cast<uint32_t *>(ws + p.off_mcnt);
  uint2 *tiebuf = reinterpret_cast<uint2 *>(ws + p.off_tie);
  uint2 *win = reinterpret_cast<uint2 *>(ws + p.off_win);
  // histograms and counters of both selections start at zero (they are contiguous in the workspace); the kernel that
  // draws the sample clears them on the side, otherwise a launch of its own does
  const size_t nz = (p.off_tie - p.off_mhist) / 4;
  if (!(p.sampling && !sample_idx)) {
    hipLaunchKernelGGL(k_zero_u32, dim3((unsigned)((nz + 1023) / 1024)), dim3(256), 0, st, mhist, nz);
    HIP_TRY(hipGetLastError());
  }

  ScanArgs a = {};
  a.X = static_cast<const char *>(c->stage1);
  a.Q = static_cast<const char *>(q1);
  a.B = B;
  a.thr = thr;
  a.cnt = cnt;
  a.surv = surv;
  a.L = p.L;
  a.cap = p.cap;

  if (p.sampling) {
    int32_t *samp = reinterpret_cast<int32_t *>(ws + p.off_sample);
    uint32_t *skeys = reinterpret_cast<uint32_t *>(ws + p.off_skeys);
    const int64_t lam_pad = (p.lambda + 31) / 32 * 32;
    const int32_t *rows = sample_idx;
    if (!rows) {
      hipLaunchKernelGGL(k_gen_sample, dim3((unsigned)((p.lambda + 255) / 256)), dim3(256), 0, st, samp, p.lambda,
                         seed, (uint64_t)c->N, mhist, nz);
      HIP_TRY(hipGetLastError());
    }
    if (!rows) rows = samp;
    static std::atomic<int> lds_raised{0};  // k_thr_select may use more dynamic LDS than the default limit
    if (p.thr_path != 3 && !lds_raised.load(std::memory_order_acquire)) {
      HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(k_thr_select), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  THR_KEYS_CAP * 4));
      lds_raised.store(1, std::memory_order_release);
    }
    ScanArgs s = a;
    s.rows = rows;
    s.x_rows = c->N;
    mol_status_t rc;
    if (p.thr_path == 2) {
      // large sample, exact-on-success mode: bracket from the first lambda0 sampled rows, then the whole sample through
      // the filtering scan (its lists share the memory of the corpus scan's lists, 16 entries each)
      float *thr0 = reinterpret_cast<float *>(ws + p.off_thr0);
      const uint32_t lcap = 16;
      {
        ProfScope ps(MOL_PROF_SAMPLE_SCORES, st);
        auto bracket = dt == MOL_F32 ? k_thr_bracket<MOL_F32> : (dt == MOL_BF16 ? k_thr_bracket<MOL_BF16> : k_thr_bracket<MOL_INT8>);
        hipLaunchKernelGGL(bracket, dim3(B), dim3(SELECT_THREADS), 0, st, s.X, s.x_rows, rows, (int)p.lambda0, s.Q,
                           (uint32_t)p.rank0, thr0);
        HIP_TRY(hipGetLastError());
        s.n_rows = p.lambda;
        s.thr = thr0;
        s.cap = lcap;
        rc = launch_scan_dt<EPI_FILTER, true>(dt, s, B, p.grid, st);
        if (rc != MOL_OK) return rc;
      }
      ProfScope ps(MOL_PROF_THRESHOLD, st);
      // room for twice the sampled scores expected above the bracket (what does not fit is dropped, see the kernel)
      const double kept = (double)p.lambda * (double)p.rank0 / (double)p.lambda0;
      uint32_t kcap = (uint32_t)(2.0 * kept) + 1024u;
      kcap = kcap > THR_KEYS_CAP ? THR_KEYS_CAP : (kcap + 1023u) & ~1023u;
      hipLaunchKernelGGL(k_thr_select, dim3(B, 2), dim3(SELECT_THREADS), (size_t)kcap * 4, st,
                         (const uint32_t *)nullptr, (int64_t)0, (int64_t)0, surv, cnt, p.L, B, lcap, kcap,
                         (uint32_t)p.rank, (uint32_t)p.rank_u, thr0, thr, win, flags, gate);
      HIP_TRY(hipGetLastError());
    } else {
      s.n_rows = p.lambda;
      s.skeys = skeys;
      s.skeys_stride = lam_pad;
      {
        ProfScope ps(MOL_PROF_SAMPLE_SCORES, st);
        rc = launch_scan_dt<EPI_KEYS, true>(dt, s, B, 0, st);
      }
      if (rc != MOL_OK) return rc;
      ProfScope ps(MOL_PROF_THRESHOLD, st);
      if (p.thr_path == 1) {
        hipLaunchKernelGGL(k_thr_select, dim3(B, 2), dim3(SELECT_THREADS), (size_t)p.lambda * 4, st, skeys, lam_pad,
                           p.lambda, (const uint2 *)nullptr, (const uint32_t *)nullptr, (int64_t)0, B, 0u,
                           (uint32_t)p.lambda, (uint32_t)p.rank, (uint32_t)p.rank_u, (const float *)nullptr, thr, win,
                           flags, gate);
        HIP_TRY(hipGetLastError());
      } else {
#ifndef MOL_THR_BLOCKS
#define MOL_THR_BLOCKS 1024
#endif
        int G = MOL_THR_BLOCKS / B;
        G = G < 1 ? 1 : (G > MOL_THR_BLOCKS / 16 ? MOL_THR_BLOCKS / 16 : G);
        const int passes = (mode & 0xff) == MOL_HINDEXER_EXACT ? MSEL_PASSES - 1 : MSEL_PASSES;
        for (int pass = 0; pass < passes; ++pass) {
          hipLaunchKernelGGL(k_thr_hist, dim3(G, B), dim3(MSEL_THREADS), 0, st, skeys, lam_pad, p.lambda, (uint32_t)p.rank,
                             (uint32_t)p.rank_u, mhist, mhist_u, B, pass);
          HIP_TRY(hipGetLastError());
        }
        hipLaunchKernelGGL(k_thr_finish, dim3(B), dim3(MSEL_THREADS), 0, st, mhist, mhist_u, B, (uint32_t)p.rank,
                           (uint32_t)p.rank_u, passes, thr, win, flags, gate);
        HIP_TRY(hipGetLastError());
      }
    }
  } else {
    hipLaunchKernelGGL(k_init_all_pass, dim3((B + 255) / 256), dim3(256), 0, st, thr, flags, gate, B);
    HIP_TRY(hipGetLastError());
  }

  a.n_rows = c->N;
  mol_status_t rc;
  {
    ProfScope ps(MOL_PROF_SCAN_FILTER, st);
    rc = launch_scan_dt<EPI_FILTER, false>(dt, a, B, p.grid, st);
  }
  if (rc != MOL_OK) return rc;

  ProfScope ps(MOL_PROF_SELECT, st);
  {
#ifndef MOL_SURV_BLOCKS
#define MOL_SURV_BLOCKS 1024
#endif
    int G = MOL_SURV_BLOCKS / B;
    G = G < 1 ? 1 : (G > MOL_SURV_BLOCKS / 32 ? MOL_SURV_BLOCKS / 32 : G);
    const uint2 *w = p.sampling ? win : nullptr;
    // no key window without a sample: three digit passes over the survivors; with windows one pass over their slices
    const int hist_passes = p.sampling ? 1 : MSEL_PASSES;
    // lanes of a wavefront per list when the lists are walked: a list holds p.cap entries at most, about a third of that
    // on average
    const bool short_lists = p.cap <= 32;
    auto hist_k = short_lists ? k_surv_hist<8> : k_surv_hist<32>;
    auto emit_k = short_lists ? k_surv_emit<8> : k_surv_emit<32>;
    for (int pass = 0; pass < hist_passes; ++pass) {
      hipLaunchKernelGGL(hist_k, dim3(G, B), dim3(MSEL_THREADS), 0, st, surv, cnt, p.L, p.cap, sstat, Kp, mhist2, w, B,
                         pass, mode, force_redo);
      HIP_TRY(hipGetLastError());
    }
    hipLaunchKernelGGL(emit_k, dim3(G, B), dim3(MSEL_THREADS), 0, st, surv, cnt, p.L, p.cap, sstat, Kp, mhist2, w, B,
                       mode, force_redo, mcnt, tiebuf, cand_idx, cand_score);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(k_surv_finish, dim3(B), dim3(MSEL_THREADS), 0, st, sstat, Kp, mhist2, w, B, tiebuf, flags, gate,
                       state, hist, cand_idx, cand_score, cand_count);
    HIP_TRY(hipGetLastError());
  }

  // the caller redoes flagged queries itself: k_surv_finish has left them with cand_count = -1 and an all -1 row
  if (defer_redo) return MOL_OK;
  // exact redo of flagged queries: 8 histogram scans and the emitting scan; each returns at once when no query is
  // flagged (k_surv_finish has set up the per-query state; the last workgroup of every scan advances it)
  a.state = state;
  a.hist = hist;
  a.gate_rw = gate;
  a.flags = flags;
  a.out_idx = cand_idx;
  a.out_score = cand_score;
  a.out_count = cand_count;
  a.Kp = Kp;
  // ~idx starts with the same 0xff digits for every item of a small corpus: those passes are not launched
  const int idx_skip = c->N <= (1 << 8) ? 3 : (c->N <= (1 << 16) ? 2 : (c->N <= (1 << 24) ? 1 : 0));
  a.idx_prefix = idx_skip ? 0xffffffffu << (32 - 8 * idx_skip) : 0u;
  for (int pass = 0; pass < 8; ++pass) {
    if (pass >= 4 && pass < 4 + idx_skip) continue;
    a.shift = 24 - 8 * (pass & 3);
    a.gate = gate + (pass < 4 ? 0 : 1);
    a.stage = pass + 1;
    if (pass < 4)
      rc = launch_scan_dt<EPI_HIST_KEY, false>(dt, a, B, 0, st);
    else
      rc = launch_scan_dt<EPI_HIST_IDX, false>(dt, a, B, 0, st);
    if (rc != MOL_OK) return rc;
  }
  a.gate = gate;
  a.paper = (mode == MOL_HINDEXER_PAPER && p.sampling) ? 1 : 0;
  rc = launch_scan_dt<EPI_FILTER_EXACT, false>(dt, a, B, 0, st);
  if (rc != MOL_OK) return rc;
  return MOL_OK;
}
