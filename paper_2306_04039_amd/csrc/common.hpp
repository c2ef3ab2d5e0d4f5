// Shared device helpers and internal structs for the retrieval library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "molret.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));

#define WAVE 64

// ---------------------------------------------------------------------------------------------
// Order-preserving map float -> uint32 (larger float <=> larger key).  -0 is folded into +0 first.
__device__ __forceinline__ uint32_t f32_to_key(float f) {
  uint32_t u = __float_as_uint(f + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_to_f32(uint32_t k) {
  uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __uint_as_float(u);
}

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
typedef float f32x2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
// two fp32 -> packed bf16 pair (round to nearest even; one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2v v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2v));
}
// a ~= hi + lo with both parts bf16: feeding both to the matrix cores keeps ~16 mantissa bits of a
__device__ __forceinline__ void split_bf16x2(float a, float b, uint32_t &hi, uint32_t &lo) {
  hi = pack_bf16x2(a, b);
  lo = pack_bf16x2(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) {
  union {
    uint4 u;
    bf16x8 b;
  } c;
  c.u = v;
  return c.b;
}

// Matrix-core results need a fixed number of idle issue slots before an ordinary vector instruction may read them; the
// hardware does not interlock this and the compiler inserts the slots itself, but it has been seen to miss the shortest
// path when a branch diamond (a conditional prefetch) sits between the last MFMA and the first read: accumulators were
// then read before the last MFMA had landed.  Called after such a diamond and before the first read, this puts the full
// wait (20 slots, enough for a 16-pass MFMA) on every path; the scheduling barriers keep MFMAs above and reads below.
__device__ __forceinline__ void mfma_settle() {
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_nop 15\n\ts_nop 3" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}

// ---- the 16-bit type of the MoL-side tensors: F16 = false bfloat16, true IEEE half (Section 4.3 serves in FP16) ----
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ f16x8 as_f16x8(uint4 v) { return __builtin_bit_cast(f16x8, v); }
template <bool F16>
__device__ __forceinline__ float dec16(uint32_t bits) {  // low 16 bits -> fp32, exact
  if constexpr (F16) return (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
  else return __uint_as_float(bits << 16);
}
__device__ __forceinline__ float dec16(uint32_t bits, bool f16) { return f16 ? dec16<true>(bits) : dec16<false>(bits); }
template <bool F16>
__device__ __forceinline__ uint32_t pack16x2(float lo, float hi) {  // round to nearest even
  if constexpr (F16) {
    f32x2v v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2v));
  } else {
    return pack_bf16x2(lo, hi);
  }
}
// a ~= hi + lo with both parts in the 16-bit type (see split_bf16x2)
template <bool F16>
__device__ __forceinline__ void split16x2(float a, float b, uint32_t &hi, uint32_t &lo) {
  hi = pack16x2<F16>(a, b);
  lo = pack16x2<F16>(a - dec16<F16>(hi & 0xffffu), b - dec16<F16>(hi >> 16));
}
template <bool F16>
__device__ __forceinline__ f32x4 mfma16_16x16x32(uint4 a, uint4 b, f32x4 c) {
  if constexpr (F16) return __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(a), as_f16x8(b), c, 0, 0, 0);
  else return __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a), as_bf16x8(b), c, 0, 0, 0);
}
template <bool F16>
__device__ __forceinline__ f32x16 mfma16_32x32x16(uint4 a, uint4 b, f32x16 c) {
  if constexpr (F16) return __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(a), as_f16x8(b), c, 0, 0, 0);
  else return __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(b), c, 0, 0, 0);
}

__device__ __forceinline__ i32x4 as_i32x4(uint4 v) {
  i32x4 r = {(int)v.x, (int)v.y, (int)v.z, (int)v.w};
  return r;
}

// 16-byte global load through a plain pointer.
__device__ __forceinline__ uint4 ld16(const void *p) { return *reinterpret_cast<const uint4 *>(p); }
// Streaming loads, for data a kernel reads once (the stage-1 table, the gathered candidate rows): marked non-temporal so
// that they do not displace what is reused.  A read-only sweep over 12.8 GB runs at 7.2 TB/s with them, 6.3 TB/s without.
typedef unsigned int mol_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int mol_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 ld16_stream(const void *p) {
  const mol_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const mol_u32x4 *>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 ld8_stream(const void *p) {
  const mol_u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const mol_u32x2 *>(p));
  return make_uint2(v.x, v.y);
}

// ---------------------------------------------------------------------------------------------
struct mol_corpus {
  int64_t N;
  int32_t d1, stage1_dtype;
  int32_t k_u, k_x, d_p, P;
  int32_t d_gu, d_gx, H, act;
  float logit_scale;
  uint32_t flags;
  int device;
  // device memory
  const void *stage1;   // [N, d1]
  const void *embs;     // bf16 [N, k_x, d_p]
  void *xi;             // bf16 [N, H]   item half of gating layer 1 (+ b1)
  void *w1c_frag;       // bf16, MFMA fragment order, [H/32][P/16][64][8]
  void *w2_frag;        // bf16, MFMA fragment order, [ceil(P/32)][H/16][64][8]
  void *w1c_frag_h;     // the same two fragment buffers as IEEE half (bf16 -> half is exact for |w| >= 2^-14); they alias
  void *w2_frag_h;      // the buffers above when the corpus is half already
  void *w1u;            // bf16 [H, d_gu] row-major (user part of layer 1)
  float *b2;            // f32 [32*ceil(P/32)] (padded with zeros)
  bool own_stage1, own_embs;
  // decomposed gate (Algorithm 1): cached item weights and the user-side MLP
  int32_t gate_form, d_hu;
  bool f16;             // the 16-bit MoL-side tensors (embeddings, gate features, weights, Xi) are IEEE half, not bfloat16
  float *xw;            // f32 [N, P]
  void *wu1, *wu2;      // bf16 [d_hu, d_gu], bf16 [P, d_hu]
  float *bu1, *bu2, *b1c;  // f32 [d_hu], f32 [P], f32 [H] (zeros when the caller gave none)
  // item embeddings generated on the fly (Section 3.1): the last k_g of the k_x item-side embeddings come from a 2-layer
  // MLP on a cached seed; embs then holds k_x - k_g embeddings per item
  int32_t k_g, d_s, d_hg;
  void *seed;              // half [N, d_s]
  void *wg1_frag, *wg2_frag;  // half, MFMA fragment order
  float *bg1, *bg2;        // f32 [d_hg], f32 [k_g * d_p]
};

// error plumbing (api.hip)
mol_status_t mol_fail(mol_status_t st, const char *fmt, ...);
#define HIP_TRY(expr)                                                                           \
  do {                                                                                          \
    hipError_t e__ = (expr);                                                                    \
    if (e__ != hipSuccess) return mol_fail(MOL_EHIP, "%s: %s", #expr, hipGetErrorString(e__)); \
  } while (0)

// per-kernel timing (api.hip): no-ops unless mol_profile_enable(1) was called
void mol_prof_begin(int slot, hipStream_t st);
void mol_prof_end(int slot, hipStream_t st);
struct ProfScope {
  int slot;
  hipStream_t st;
  ProfScope(int s, hipStream_t t) : slot(s), st(t) { mol_prof_begin(slot, st); }
  ~ProfScope() { mol_prof_end(slot, st); }
};

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- launchers implemented in the kernel files ------------------------------------------------
// stage1.hip
struct HindexerPlan {
  bool sampling;       // false: every item passes (threshold -inf)
  int64_t lambda;      // sample size actually used
  int64_t rank;        // threshold rank inside the sample (1-based from the largest)
  int64_t grid;        // workgroups of the list-writing scans
  int64_t L;           // survivor lists per query (8 per workgroup)
  int64_t cap;         // capacity of one survivor list
  // how the threshold is taken from the sample: 0 no sampling, 1 the sampled scores fit one workgroup's LDS,
  // 2 large sample, bracket from its first lambda0 rows then a filtering scan over all of it (the threshold may then lie
  // below the rank-th sampled score, never above: exact-on-success mode only), 3 large sample, digit passes over the
  // B x lambda score matrix (exact rank)
  int thr_path;
  int64_t lambda0;     // path 2: rows of the bracketing part of the sample
  int64_t rank0;       // path 2: rank of the bracket inside that part
  int64_t rank_u;      // rank of the upper end of the key window inside the sample (0: none)
  // workspace offsets (bytes)
  size_t off_sample, off_skeys, off_thr, off_thr0, off_win, off_count, off_flags, off_sstat, off_surv, off_mhist, off_mcnt,
      off_tie, off_hist, off_state, total;
};
mol_status_t hindexer_plan(const mol_corpus *c, int B, int Kp, int64_t lambda, int mode, HindexerPlan *p);
mol_status_t hindexer_run(const mol_corpus *c, const void *q1, int B, int Kp, const int32_t *sample_idx,
                          uint64_t seed, int mode, const HindexerPlan &p, int32_t *cand_idx, float *cand_score,
                          int32_t *cand_count, char *ws, hipStream_t st);
// pack.hip
mol_status_t launch_item_gate_cache(const mol_corpus *c, const void *item_gate, const void *w1x_rowmajor,
                                    const float *b1, hipStream_t st);
// mol.hip
// U [B, H] and (decomposed gate) UW [B, P]: the per-query inputs of the scoring kernel
// UP [B, H] (may be NULL): U as half head | half remainder << 16, read by the exhaustive fast form only
mol_status_t launch_user_gate(const mol_corpus *c, const void *user_gate, int B, float *U, float *UW, uint32_t *UP,
                              hipStream_t st);
mol_status_t launch_mol_score(const mol_corpus *c, const void *user_embs, const float *U, const float *UW,
                              const uint32_t *UP, int B, const int32_t *cand_idx, const int32_t *cand_count, int64_t Kp,
                              float *scores, hipStream_t st);
bool mol_exh_fast_form(const mol_corpus *c);
bool mol_gen_shape_supported(int k_u, int k_x, int d_p, int H, int k_g, int d_s, int d_hg);
mol_status_t launch_gather_items(const mol_corpus *c, const int32_t *cand_idx, int B, int64_t Kp, void *out, hipStream_t st);
// select.hip
size_t final_topk_workspace_bytes(int B, int64_t Kp, int k);
mol_status_t launch_final_topk(const float *scores, const int32_t *cand_idx, const int32_t *cand_count, int B, int64_t Kp,
                               int k, int32_t *out_idx, float *out_score, char *ws, hipStream_t st);
