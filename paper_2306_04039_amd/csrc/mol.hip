// Stage 2, Mixture of Logits (Section 3, Algorithm 1), one fused kernel per call.
//
// A wavefront scores tiles of 32 candidates of one query.  Per tile:
//   A. component logits cl[c, ku*k_x + kx] = logit_scale * <F[b,ku], G[n_c,kx]>  (Eq. 6, Eq. 9): candidate rows are
//      gathered from the item cache straight into MFMA operand registers (16x16x32 bf16, rows = (candidate, kx),
//      columns = ku); the fp32 result goes to a small LDS tile, already in the permuted (candidate, P) order that
//      Algorithm 1 produces with view/permute, so the permute costs nothing (Section 4.2).
//   B. gating layer 1, transposed: pre^T[h, c] = W1c[h, :] . cl[c, :] on 32x32x16 MFMA, plus the per-query user
//      part U[b, h] and the cached item part Xi[n_c, h] (Section 3.2 decomposition), activation in registers.
//   C. gating layer 2, transposed: z^T[p, c] = W2[p, :] . hid[c, :]; the layer-1 accumulators are exactly the
//      B-operand of this product (same lane = same candidate), so hidden activations never leave registers.
//   D. softmax over the P components and phi = sum_p pi_p * cl_p (Eq. 3) with the fp32 logits from the LDS tile;
//      each candidate's P values sit in two lanes (lane, lane^32).
// Nothing but the final score is written to HBM (the fusion Section 4.2 argues for).
// The weights are bf16 by contract; the activations that feed the matrix cores (logits, hidden units) are fp32
// values, so each is split into a bf16 head and a bf16 remainder and multiplied twice: the gate then sees them
// to ~16 mantissa bits, which keeps phi within 2e-3 of the fp64 definition even for large logit scales.
#include <math.h>

#include <mutex>

#include "common.hpp"

namespace {

struct MolArgs {
  const char *embs;      // bf16 [N, K_X, D_P]
  const char *xi;        // bf16 [N, H]
  const char *w1c_frag;  // bf16 fragments
  const char *w2_frag;   // bf16 fragments
  const float *b2;       // f32 [32*PT]
  const char *F;         // bf16 [B, K_U, D_P]
  const float *U;        // f32 [B, H]   per-query additive term of layer 1 (user part; for the decomposed gate just b1)
  const float *xw;       // decomposed gate: f32 [N, P] cached item weights
  const float *UW;       // decomposed gate: f32 [B, P] user weights
  const char *w1c_frag_h;   // the layer-1 / layer-2 fragments as IEEE half (exhaustive fast path)
  const char *w2_frag_h;
  // item embeddings generated on the fly (Section 3.1): seed vectors and the generator MLP, all IEEE half
  const char *seed;         // half [N, D_S]
  const char *wg1_frag;     // half, MFMA fragment order [D_HG/16][D_S/32][64][8]
  const char *wg2_frag;     // half, MFMA fragment order [K_G*D_P/16][D_HG/32][64][8] (k-slots permuted, see pack)
  const float *bg1, *bg2;   // f32 [D_HG], f32 [K_G*D_P]
  const uint32_t *UP;       // [B][H/32][64]: U[b, 32 mt + l] as a half head | half remainder << 16 at [b][mt][l], l < 32,
                            // zeros at l >= 32 (the A operand of the extra k-step, one word per lane; exhaustive fast path)
  const int32_t *cand;   // [B, Kp] or nullptr (exhaustive: candidate c is item c)
  const int32_t *cand_count;  // [B] or nullptr: only the first cand_count[b] slots of row b are candidates
  float *scores;         // [B, Kp]
  int64_t Kp;            // row length of cand / scores
  int64_t N;
  int B;
  int act;
  float logit_scale;
};

template <int K_U, int K_X, int D_P, int H>
struct MolShape {
  static constexpr int P = K_U * K_X;
  static constexpr int MT = H / 32;          // row tiles of layer 1 (hidden units)
  static constexpr int S1 = P / 16;          // k-steps of layer 1
  static constexpr int PT = (P + 31) / 32;   // row tiles of layer 2 (components)
  static constexpr int S2 = H / 16;          // k-steps of layer 2
  static constexpr int SA = D_P / 32;        // k-steps of the component-logit product
  static constexpr int CPR = 16 / K_X;       // candidates per 16-row MFMA tile
  static constexpr int RT = 32 / CPR;        // 16-row tiles per 32 candidates
  static constexpr int CLS = P + 4;          // LDS row stride of the logit tile (floats)
  static constexpr int W1B = MT * S1 * 1024; // bytes
  static constexpr int W2B = PT * S2 * 1024;
  static constexpr int WAVE_FLOATS = 32 * CLS + H + 32 * PT;  // logit tile, U[b], user weights (decomposed gate)
  static constexpr size_t LDS = W1B + W2B + PT * 32 * 4 + 4 * WAVE_FLOATS * 4;
};

// Generator of on-the-fly item embeddings (Section 3.1): K_G of the K_X item-side embeddings come from a 2-layer MLP on a
// cached seed of D_S numbers (hidden width D_HG) instead of the cache.  K_G = 0: none.
template <int K_G, int D_P, int D_S, int D_HG>
struct GenShape {
  static constexpr int UT = D_HG / 16;            // 16-row tiles of layer 1 (hidden units)
  static constexpr int SG1 = D_S / 32;            // k-steps of layer 1
  static constexpr int FT = K_G * D_P / 16;       // 16-row tiles of layer 2 (output features)
  static constexpr int SG2 = D_HG / 32;           // k-steps of layer 2
  static constexpr int W1B = K_G ? UT * SG1 * 1024 : 0;  // bytes of the fragment buffers
  static constexpr int W2B = K_G ? FT * SG2 * 1024 : 0;
  static constexpr int BIAS_FLOATS = K_G ? D_HG + K_G * D_P : 0;
  static constexpr size_t LDS = W1B + W2B + BIAS_FLOATS * 4;
};

__device__ __forceinline__ float act_fn(float x, int act) {
  return act == MOL_ACT_RELU ? fmaxf(x, 0.f) : x / (1.f + __expf(-x));
}

// Reductions over the two halves of a wavefront (lane and lane ^ 32) without a trip through LDS: the row swap leaves the
// lower half's value in one register and the upper half's in the other, in every lane.
__device__ __forceinline__ float half_swap_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_swap_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// x + the value of lane ^ 16, in every lane (rows of 16 lanes swapped in pairs)
__device__ __forceinline__ float quarter_swap_sum(float x) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// EXH = false: tiles of 32 candidates of one query (cand list or not), every tile gathers its own rows.
// EXH = true : exhaustive scoring (every item for every query).  A wavefront takes a block of 32 consecutive items,
//              loads their rows and cached gate halves into registers ONCE and walks a chunk of queries over them, so
//              the item tensors are read once per query chunk instead of once per query (the per-query form moves
//              B x the corpus through L2 and is bound by that, not by the matrix cores).
#define MOL_QCHUNK 256
#ifndef MOL_PF_ROWS
#define MOL_PF_ROWS 4  // row-tile loads of the next tile started before the gating stages (registers stay live there)
#endif
#ifndef MOL_PF_XI
#define MOL_PF_XI 0    // also start the next tile's cached item-gate loads early
#endif
// With MOL_PF_XI = 1 a conditional load would sit between the layer-2 MFMA chain and the first read of its accumulators
// (the branch pattern after which matrix-core results were once read too early in the corpus scan): not supported.
static_assert(MOL_PF_XI == 0, "MOL_PF_XI = 1 needs mfma_settle() after the prefetch");
// FORM = 0: the gate is one 2-layer MLP on [cl | user feature | item feature] (first layer split into a cross part on the
//           matrix cores, U[b] and the cached Xi[n]).
// FORM = 1: Algorithm 1's decomposedGating: z = SiLU(uw[b] * xw[n] + crossMLP(cl)), uw per query, xw cached per item.
// F16: the 16-bit inputs are IEEE half instead of bfloat16 (same layouts, the half-precision MFMA forms).
// K_G > 0: the last K_G of the K_X item-side embeddings are generated per candidate inside the kernel (GenShape), the
// item cache then holds K_X - K_G embeddings per item; such instances run 8 wavefronts per workgroup so that the
// larger set of weights in LDS is shared by as many wavefronts per compute unit as before.
template <int K_U, int K_X, int D_P, int H, bool EXH, int FORM, bool F16, int K_G = 0, int D_S = 32, int D_HG = 64>
__global__ __launch_bounds__(K_G ? 512 : 256) void k_mol_score(MolArgs a) {
  using S = MolShape<K_U, K_X, D_P, H>;
  using GS = GenShape<K_G, D_P, D_S, D_HG>;
  constexpr int P = S::P, MT = S::MT, S1 = S::S1, PT = S::PT, S2 = S::S2, SA = S::SA, CPR = S::CPR, RT = S::RT,
                CLS = S::CLS;
  constexpr int NW = K_G ? 8 : 4;     // wavefronts per workgroup
  constexpr int NT = NW * 64;
  constexpr int K_C = K_X - K_G;      // cached item-side embeddings per item
  static_assert(!(EXH && K_G), "generated embeddings use the per-candidate form");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char *w1s = smem;
  char *w2s = smem + S::W1B;
  char *wg1s = smem + S::W1B + S::W2B;
  char *wg2s = wg1s + GS::W1B;
  float *bgs = reinterpret_cast<float *>(wg2s + GS::W2B);   // [D_HG] then [K_G * D_P]
  float *b2s = bgs + GS::BIAS_FLOATS;
  const int wv = threadIdx.x >> 6;
  float *cl = b2s + PT * 32 + wv * S::WAVE_FLOATS;  // [32][CLS]
  float *Us = cl + 32 * CLS;                        // [H]
  float *UWs = Us + H;                              // [32 * PT] (FORM 1)

  // stage the weight fragments once per workgroup
  for (int i = threadIdx.x; i < S::W1B / 16; i += NT)
    reinterpret_cast<uint4 *>(w1s)[i] = reinterpret_cast<const uint4 *>(a.w1c_frag)[i];
  for (int i = threadIdx.x; i < S::W2B / 16; i += NT)
    reinterpret_cast<uint4 *>(w2s)[i] = reinterpret_cast<const uint4 *>(a.w2_frag)[i];
  for (int i = threadIdx.x; i < PT * 32; i += NT) b2s[i] = a.b2[i];
  if constexpr (K_G > 0) {
    for (int i = threadIdx.x; i < GS::W1B / 16; i += NT)
      reinterpret_cast<uint4 *>(wg1s)[i] = reinterpret_cast<const uint4 *>(a.wg1_frag)[i];
    for (int i = threadIdx.x; i < GS::W2B / 16; i += NT)
      reinterpret_cast<uint4 *>(wg2s)[i] = reinterpret_cast<const uint4 *>(a.wg2_frag)[i];
    for (int i = threadIdx.x; i < D_HG; i += NT) bgs[i] = a.bg1[i];
    for (int i = threadIdx.x; i < K_G * D_P; i += NT) bgs[D_HG + i] = a.bg2[i];
  }
  __syncthreads();

  const int lane = threadIdx.x & 63;
  const int c = lane & 31, h = lane >> 5;     // 32x32 tiles: candidate / half
  const int r16 = lane & 15, g = lane >> 4;   // 16x16 tiles: row (or ku column) / k-group
  const int64_t tpq = (a.Kp + 31) >> 5;       // tiles per query
  const int64_t ntiles = tpq * a.B;
  const int64_t wave = (int64_t)blockIdx.x * NW + wv;
  const int64_t nwaves = (int64_t)gridDim.x * NW;

  int cur_b = -1;
  uint4 Ff[SA];
  uint4 Ffp[K_G ? SA : 1];  // K_G > 0: the user embeddings as halves in the k order of the generated rows
  uint4 sd[K_G ? 2 : 1][K_G ? GenShape<K_G, D_P, D_S, D_HG>::SG1 : 1];  // K_G > 0: the candidates' seeds (16 per half-tile)
  constexpr int PD = RT < 8 ? RT : 8;
  uint4 A[PD][SA];
  uint2 xi[MT][4];      // FORM 0: cached item half of layer 1 (bf16 x 4)
  float4 xwv[PT][4];    // FORM 1: cached item weights of this lane's components
  int idx = -1, idxc = 0;
  bool ok = false;
  const int64_t n_qch = EXH ? (a.B + MOL_QCHUNK - 1) / MOL_QCHUNK : 1;
  const int64_t ntasks = EXH ? tpq * n_qch : ntiles;
  // !EXH: the gathers of a tile are started while the previous tile is still in its gating stages (the row registers
  // are free after stage A, the item-gate registers after stage C), so a wavefront always has loads in flight.
  // idx_n / idxc_n: this lane's candidate of the next tile; primed: the current tile's gathers were started early.
  auto task_cand = [&](int64_t t) -> int {
    const int tb = (int)(t / tpq);
    const int64_t tc = ((t % tpq) << 5) + c;
    const int64_t row_len = a.cand_count ? (int64_t)a.cand_count[tb] : a.Kp;
    return tc < a.Kp && tc < row_len ? (a.cand ? a.cand[(size_t)tb * a.Kp + tc] : (int)tc) : -1;
  };
  int idx_n = -1, idxc_n = 0;
  bool primed = false;
  if (!EXH && wave < ntasks) idx_n = task_cand(wave);
  for (int64_t task = wave; task < ntasks; task += nwaves) {
   const int b_lo = EXH ? (int)(task % n_qch) * MOL_QCHUNK : 0;
   const int b_hi = EXH ? (b_lo + MOL_QCHUNK < a.B ? b_lo + MOL_QCHUNK : a.B) : 1;
   for (int bq = b_lo; bq < b_hi; ++bq) {
    int b;
    int64_t c0;
    if (EXH) {
      b = bq;
      c0 = (task / n_qch) << 5;
    } else {
      b = (int)(task / tpq);
      c0 = (task % tpq) << 5;
    }
    const bool new_items = !EXH || bq == b_lo;
    const int64_t cpos = c0 + c;
    const bool have_next = !EXH && task + nwaves < ntasks;
    if (new_items) {
      if (EXH) {
        idx = -1;
        if (cpos < a.Kp) idx = a.cand ? a.cand[(size_t)b * a.Kp + cpos] : (int)cpos;
      } else {
        idx = idx_n;
        idx_n = have_next ? task_cand(task + nwaves) : -1;
      }
      ok = idx >= 0 && idx < a.N;
      idxc = ok ? idx : 0;
    }

    if (b != cur_b) {
      cur_b = b;
#pragma unroll
      for (int s = 0; s < SA; ++s)
        Ff[s] = (r16 < K_U) ? ld16(a.F + ((size_t)(b * K_U + r16) * D_P + 32 * s + 8 * g) * 2) : make_uint4(0, 0, 0, 0);
      if constexpr (K_G > 0) {
        // k-slots e < 4 of group g hold d = 32 s + 4 g + e, slots e >= 4 hold d = 32 s + 16 + 4 g + (e - 4): the order in
        // which the generator leaves its output in registers (two 16-row result tiles side by side)
#pragma unroll
        for (int s = 0; s < SA; ++s) {
          uint2 lo = make_uint2(0, 0), hi = make_uint2(0, 0);
          if (r16 < K_U) {
            const char *fp = a.F + ((size_t)(b * K_U + r16) * D_P + 32 * s + 4 * g) * 2;
            lo = *reinterpret_cast<const uint2 *>(fp);
            hi = *reinterpret_cast<const uint2 *>(fp + 32);
          }
          if constexpr (F16) {
            Ffp[s] = make_uint4(lo.x, lo.y, hi.x, hi.y);
          } else {  // bfloat16 -> half (exact for normal halves)
            Ffp[s] = make_uint4(pack16x2<true>(dec16<false>(lo.x & 0xffffu), dec16<false>(lo.x >> 16)),
                                pack16x2<true>(dec16<false>(lo.y & 0xffffu), dec16<false>(lo.y >> 16)),
                                pack16x2<true>(dec16<false>(hi.x & 0xffffu), dec16<false>(hi.x >> 16)),
                                pack16x2<true>(dec16<false>(hi.y & 0xffffu), dec16<false>(hi.y >> 16)));
          }
        }
      }
      for (int i = lane; i < H; i += 64) Us[i] = a.U[(size_t)b * H + i];
      if constexpr (FORM == 1)
        for (int i = lane; i < 32 * PT; i += 64) UWs[i] = i < P ? a.UW[(size_t)b * P + i] : 0.f;
    }

    // item half of layer 1 for this lane's candidate: hidden units 32*mt + 8*q + 4*h + {0..3}
    auto load_xi = [&](int item) {
      if constexpr (FORM == 0) {
        const char *xp = a.xi + ((size_t)item * H + 4 * h) * 2;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int q = 0; q < 4; ++q) xi[mt][q] = *reinterpret_cast<const uint2 *>(xp + (32 * mt + 8 * q) * 2);
      } else {
        const float *xp = a.xw + (size_t)item * P + 4 * h;  // components 32*pt + 8*q + 4*h + {0..3}
#pragma unroll
        for (int pt = 0; pt < PT; ++pt)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            xwv[pt][q] = (32 * pt + 8 * q < P) ? *reinterpret_cast<const float4 *>(xp + 32 * pt + 8 * q)
                                               : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    };
    if (new_items && !(primed && MOL_PF_XI)) load_xi(idxc);

    // ---- A: component logits -> LDS tile --------------------------------------------------------------
    auto load_rows = [&](uint4(&dst)[SA], int rt, int item = -1) {
      const int ci = rt * CPR + r16 / K_X;
      const int nidx = __shfl(item < 0 ? idxc : item, ci);
      const int kx = r16 % K_X;
      const char *rowp = a.embs + (((size_t)nidx * K_C + (kx < K_C ? kx : 0)) * D_P + 8 * g) * 2;
#pragma unroll
      for (int s = 0; s < SA; ++s) dst[s] = (K_G == 0 || kx < K_C) ? ld16(rowp + 64 * s) : make_uint4(0, 0, 0, 0);
    };
    constexpr int PFR = MOL_PF_ROWS < PD ? MOL_PF_ROWS : PD;
    // seeds of the tile's candidates (generated embeddings): fetched with the previous tile's prefetch when there was one
    auto load_seeds = [&](int item) {
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        const int gidx = __shfl(item, 16 * hf + r16);
#pragma unroll
        for (int s = 0; s < GS::SG1; ++s) sd[hf][s] = ld16(a.seed + ((size_t)gidx * D_S + 32 * s + 8 * g) * 2);
      }
    };
    if constexpr (K_G > 0) {
      if (!primed) load_seeds(idxc);
    }
    if (EXH ? (new_items || RT > PD) : true) {
#pragma unroll
      for (int i = 0; i < PD; ++i)
        if (EXH || i >= PFR || !primed) load_rows(A[i], i);
    }
    // ---- G: the generated item embeddings of the tile's 32 candidates, 16 at a time, all in registers -------------------
    // 16x16x32 half MFMAs with the weights as the row operand and the candidates as columns: lane (r16, g) ends up with
    // rows 4 g + j of every 16-row result tile for candidate r16, which -- two tiles side by side -- is an 8-value k
    // group of the next product's column operand, in the k order the weight fragments / Ffp were laid out for.
    uint4 Agen[K_G ? 2 : 1][K_G ? K_G : 1][SA];
    if constexpr (K_G > 0) {
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        uint4 hb[GS::SG2];   // hidden units as halves: the column operand of layer 2
        uint32_t *hw = reinterpret_cast<uint32_t *>(hb);
#pragma unroll
        for (int ut = 0; ut < GS::UT; ++ut) {
          const float4 bi = *reinterpret_cast<const float4 *>(&bgs[16 * ut + 4 * g]);
          f32x4 acc = {bi.x, bi.y, bi.z, bi.w};
#pragma unroll
          for (int s = 0; s < GS::SG1; ++s)
            acc = mfma16_16x16x32<true>(*reinterpret_cast<const uint4 *>(wg1s + ((ut * GS::SG1 + s) * 64 + lane) * 16), sd[hf][s], acc);
          // tile ut -> words 2 (ut % 2), 2 (ut % 2) + 1 of k-step ut / 2
          hw[4 * (ut >> 1) + 2 * (ut & 1)] = pack16x2<true>(act_fn(acc[0], a.act), act_fn(acc[1], a.act));
          hw[4 * (ut >> 1) + 2 * (ut & 1) + 1] = pack16x2<true>(act_fn(acc[2], a.act), act_fn(acc[3], a.act));
        }
#pragma unroll
        for (int kg = 0; kg < K_G; ++kg) {
          f32x4 ev[D_P / 16];
          float ss = 0.f;
#pragma unroll
          for (int dt = 0; dt < D_P / 16; ++dt) {
            const int ft = kg * (D_P / 16) + dt;
            const float4 bi = *reinterpret_cast<const float4 *>(&bgs[D_HG + 16 * ft + 4 * g]);
            f32x4 acc = {bi.x, bi.y, bi.z, bi.w};
#pragma unroll
            for (int s = 0; s < GS::SG2; ++s)
              acc = mfma16_16x16x32<true>(*reinterpret_cast<const uint4 *>(wg2s + ((ft * GS::SG2 + s) * 64 + lane) * 16), hb[s], acc);
            ev[dt] = acc;
            ss += (acc[0] * acc[0] + acc[1] * acc[1]) + (acc[2] * acc[2] + acc[3] * acc[3]);
          }
          // L2 norm over the D_P values of (candidate, kg): they sit in the four lanes r16 + 16 g
          ss = quarter_swap_sum(ss);
          ss = half_swap_sum(ss);
          const float inv = 1.0f / fmaxf(sqrtf(ss), 1e-12f);
#pragma unroll
          for (int sa = 0; sa < SA; ++sa)
            Agen[hf][kg][sa] = make_uint4(pack16x2<true>(ev[2 * sa][0] * inv, ev[2 * sa][1] * inv),
                                          pack16x2<true>(ev[2 * sa][2] * inv, ev[2 * sa][3] * inv),
                                          pack16x2<true>(ev[2 * sa + 1][0] * inv, ev[2 * sa + 1][1] * inv),
                                          pack16x2<true>(ev[2 * sa + 1][2] * inv, ev[2 * sa + 1][3] * inv));
        }
      }
    }

#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < SA; ++s)
        acc = mfma16_16x16x32<F16>(A[rt % PD][s], Ff[s], acc);
      if (rt + PD < RT) load_rows(A[rt % PD], rt + PD);
      // acc[j]: row 4*g + j of the tile = (candidate rt*CPR + (4g+j)/K_X, kx (4g+j)%K_X); column ku = r16
      if (r16 < K_U) {
        if constexpr (K_X % 4 == 0) {
          float4 v = make_float4(acc[0] * a.logit_scale, acc[1] * a.logit_scale, acc[2] * a.logit_scale,
                                 acc[3] * a.logit_scale);
          *reinterpret_cast<float4 *>(&cl[(rt * CPR + (4 * g) / K_X) * CLS + r16 * K_X + (4 * g) % K_X]) = v;
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            cl[(rt * CPR + (4 * g + j) / K_X) * CLS + r16 * K_X + (4 * g + j) % K_X] = acc[j] * a.logit_scale;
        }
      }
    }
    if constexpr (K_G > 0) {
      // logits of the generated embeddings: rows = 16 candidates, columns = ku; they take places K_C .. K_X - 1 of each
      // user's group of K_X components (after the cached tiles above have written those places with zeros)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int kg = 0; kg < K_G; ++kg) {
          f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int sa = 0; sa < SA; ++sa) acc = mfma16_16x16x32<true>(Agen[hf][kg][sa], Ffp[sa], acc);
          const float v0 = acc[0] * a.logit_scale, v1 = acc[1] * a.logit_scale, v2 = acc[2] * a.logit_scale,
                      v3 = acc[3] * a.logit_scale;  // read before the branch
          if (r16 < K_U) {
            float *dst = &cl[(16 * hf + 4 * g) * CLS + r16 * K_X + K_C + kg];
            dst[0] = v0;
            dst[CLS] = v1;
            dst[2 * CLS] = v2;
            dst[3 * CLS] = v3;
          }
        }
    }
    if (have_next) {  // the row registers are free: start the next tile's first rows
      idxc_n = (idx_n >= 0 && idx_n < a.N) ? idx_n : 0;
#pragma unroll
      for (int i = 0; i < PFR; ++i) load_rows(A[i], i, idxc_n);
      if constexpr (K_G > 0) load_seeds(idxc_n);  // the generator has consumed this tile's seeds
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- B: layer 1 (transposed): acc1[mt][j] = pre[h = 32mt + 8(j/4) + 4h + j%4][candidate c] ---------
    f32x16 acc1[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc1[mt][j] = 0.f;
#pragma unroll
    for (int s = 0; s < S1; ++s) {
      const float4 lo = *reinterpret_cast<const float4 *>(&cl[c * CLS + 16 * s + 8 * h]);
      const float4 hi = *reinterpret_cast<const float4 *>(&cl[c * CLS + 16 * s + 8 * h + 4]);
      uint4 bh, bl;
      split16x2<F16>(lo.x, lo.y, bh.x, bl.x);
      split16x2<F16>(lo.z, lo.w, bh.y, bl.y);
      split16x2<F16>(hi.x, hi.y, bh.z, bl.z);
      split16x2<F16>(hi.z, hi.w, bh.w, bl.w);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const uint4 af = *reinterpret_cast<const uint4 *>(w1s + ((mt * S1 + s) * 64 + lane) * 16);
        acc1[mt] = mfma16_32x32x16<F16>(af, bl, acc1[mt]);
        acc1[mt] = mfma16_32x32x16<F16>(af, bh, acc1[mt]);
      }
    }

    // ---- C: activation, then layer 2 (transposed): acc2[pt][j] = z[p = 32pt + 8(j/4) + 4h + j%4][c] -----
    f32x16 acc2[PT];
#pragma unroll
    for (int pt = 0; pt < PT; ++pt)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc2[pt][j] = 0.f;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int qq = 0; qq < 2; ++qq) {
        float hid[8];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const int q = 2 * qq + t;
          const float4 u4 = *reinterpret_cast<const float4 *>(&Us[32 * mt + 8 * q + 4 * h]);
          if constexpr (FORM == 0) {
            const uint2 x = xi[mt][q];
            hid[4 * t + 0] = act_fn(acc1[mt][4 * q + 0] + u4.x + dec16<F16>(x.x & 0xffffu), a.act);
            hid[4 * t + 1] = act_fn(acc1[mt][4 * q + 1] + u4.y + dec16<F16>(x.x >> 16), a.act);
            hid[4 * t + 2] = act_fn(acc1[mt][4 * q + 2] + u4.z + dec16<F16>(x.y & 0xffffu), a.act);
            hid[4 * t + 3] = act_fn(acc1[mt][4 * q + 3] + u4.w + dec16<F16>(x.y >> 16), a.act);
          } else {  // the cross MLP sees the logits only; u4 carries its bias
            hid[4 * t + 0] = act_fn(acc1[mt][4 * q + 0] + u4.x, a.act);
            hid[4 * t + 1] = act_fn(acc1[mt][4 * q + 1] + u4.y, a.act);
            hid[4 * t + 2] = act_fn(acc1[mt][4 * q + 2] + u4.z, a.act);
            hid[4 * t + 3] = act_fn(acc1[mt][4 * q + 3] + u4.w, a.act);
          }
        }
        uint4 bh, bl;
        split16x2<F16>(hid[0], hid[1], bh.x, bl.x);
        split16x2<F16>(hid[2], hid[3], bh.y, bl.y);
        split16x2<F16>(hid[4], hid[5], bh.z, bl.z);
        split16x2<F16>(hid[6], hid[7], bh.w, bl.w);
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
          const uint4 af = *reinterpret_cast<const uint4 *>(w2s + ((pt * S2 + mt * 2 + qq) * 64 + lane) * 16);
          acc2[pt] = mfma16_32x32x16<F16>(af, bl, acc2[pt]);
          acc2[pt] = mfma16_32x32x16<F16>(af, bh, acc2[pt]);
        }
      }
    }

    if (have_next && MOL_PF_XI) load_xi(idxc_n);  // the item-gate registers are free: the next tile's cached gate halves
    primed = have_next;

    // ---- D: softmax over components and the weighted sum --------------------------------------------------
    float m = -INFINITY;
#pragma unroll
    for (int pt = 0; pt < PT; ++pt)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (32 * pt + 8 * q < P) {  // P is a multiple of 16: a group of 8 is all valid or all padding
          const float4 b4 = *reinterpret_cast<const float4 *>(&b2s[32 * pt + 8 * q + 4 * h]);
          acc2[pt][4 * q + 0] += b4.x;
          acc2[pt][4 * q + 1] += b4.y;
          acc2[pt][4 * q + 2] += b4.z;
          acc2[pt][4 * q + 3] += b4.w;
          if constexpr (FORM == 1) {  // combineFn: uw * xw + cw, then SiLU (Section 3.4)
            const float4 u4 = *reinterpret_cast<const float4 *>(&UWs[32 * pt + 8 * q + 4 * h]);
            const float4 x4 = xwv[pt][q];
            acc2[pt][4 * q + 0] = act_fn(fmaf(u4.x, x4.x, acc2[pt][4 * q + 0]), MOL_ACT_SILU);
            acc2[pt][4 * q + 1] = act_fn(fmaf(u4.y, x4.y, acc2[pt][4 * q + 1]), MOL_ACT_SILU);
            acc2[pt][4 * q + 2] = act_fn(fmaf(u4.z, x4.z, acc2[pt][4 * q + 2]), MOL_ACT_SILU);
            acc2[pt][4 * q + 3] = act_fn(fmaf(u4.w, x4.w, acc2[pt][4 * q + 3]), MOL_ACT_SILU);
          }
#pragma unroll
          for (int i = 0; i < 4; ++i) m = fmaxf(m, acc2[pt][4 * q + i]);
        }
      }
    m = fmaxf(m, __shfl_xor(m, 32));
    float den = 0.f, num = 0.f;
#pragma unroll
    for (int pt = 0; pt < PT; ++pt)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (32 * pt + 8 * q < P) {
          const float4 c4 = *reinterpret_cast<const float4 *>(&cl[c * CLS + 32 * pt + 8 * q + 4 * h]);
          const float e0 = __expf(acc2[pt][4 * q + 0] - m), e1 = __expf(acc2[pt][4 * q + 1] - m),
                      e2 = __expf(acc2[pt][4 * q + 2] - m), e3 = __expf(acc2[pt][4 * q + 3] - m);
          den += (e0 + e1) + (e2 + e3);
          num += (e0 * c4.x + e1 * c4.y) + (e2 * c4.z + e3 * c4.w);
        }
      }
    den += __shfl_xor(den, 32);
    num += __shfl_xor(num, 32);
    if (h == 0 && cpos < a.Kp) a.scores[(size_t)b * a.Kp + cpos] = ok ? num / den : -INFINITY;
    // the next tile overwrites the LDS logit tile: all lanes must be done reading it
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
   }
  }
}

// Exhaustive scoring, fast form (cand_idx = NULL, concatenated gate, ReLU, shapes whose item tile fits registers).
// Every (query, item) pair costs the same arithmetic, so what bounds this kernel is instruction issue -- matrix-core
// and vector -- not memory (Section 4.2: the non-GEMM operators dominate once the GEMMs are on the matrix cores).
// Against the general kernel above it
//   * keeps a block of 32 items (rows and decoded gate halves) in registers and walks a chunk of queries over it;
//   * scores 16 / K_U queries per component-logit MFMA (the 16 columns hold (query, ku) pairs instead of K_U columns
//     and padding), the logits of the group go to an LDS tile per query;
//   * runs both gating layers on the half-precision MFMA forms: the bf16 weights convert to half exactly (pack does it
//     once), logits and hidden units are rounded once to half (11 significant bits) instead of being split into two
//     bf16 parts -- one MFMA and one conversion per operand instead of two MFMAs and a split;
//   * lets the matrix cores add what is constant over a tile: the cached item half Xi[n] and b2 enter as the MFMA's
//     initial accumulators, the user half U[b] as one more k-step (a half head + remainder against a column of ones);
//   * applies ReLU on packed halves (it commutes with the rounding).
// registers one lane holds for a whole item block (decoded gate halves, layer-1 accumulators, rows, layer-2 accumulators
// and bias): shapes beyond 170 of them get the whole register file (one wavefront per SIMD), the others share it in two
template <int K_U, int K_X, int D_P, int H>
constexpr int exh_min_waves() {
  using S = MolShape<K_U, K_X, D_P, H>;
  return (S::MT * 32 + S::RT * S::SA * 4 + S::PT * 32 > 170) ? 1 : 2;
}

template <int K_U, int K_X, int D_P, int H, bool F16>
__global__ __launch_bounds__(256, (exh_min_waves<K_U, K_X, D_P, H>())) void k_mol_exh(MolArgs a) {
  using S = MolShape<K_U, K_X, D_P, H>;
  constexpr int P = S::P, MT = S::MT, S1 = S::S1, PT = S::PT, S2 = S::S2, SA = S::SA, CPR = S::CPR, RT = S::RT,
                CLS = S::CLS;
  constexpr int QPM = 16 / K_U;  // queries per component-logit MFMA
  static_assert(RT <= 8, "the item tile must fit the register file");
  // small gates keep their weight fragments in registers for the whole kernel (each is read once per query otherwise,
  // and LDS bandwidth is a co-limit of this kernel); larger ones stage them in LDS
  constexpr bool WREG = MT * S1 + PT * S2 <= 8;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char *w1s = smem;
  char *w2s = smem + S::W1B;
  const int wv = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  float *cl = reinterpret_cast<float *>(smem + (WREG ? 0 : S::W1B + S::W2B)) + wv * (QPM * 32 * CLS);  // [QPM][32][CLS]
  uint4 w1r[WREG ? MT * S1 : 1], w2r[WREG ? PT * S2 : 1];
  if constexpr (WREG) {
#pragma unroll
    for (int i = 0; i < MT * S1; ++i) w1r[i] = reinterpret_cast<const uint4 *>(a.w1c_frag_h)[i * 64 + lane];
#pragma unroll
    for (int i = 0; i < PT * S2; ++i) w2r[i] = reinterpret_cast<const uint4 *>(a.w2_frag_h)[i * 64 + lane];
  } else {
    for (int i = threadIdx.x; i < S::W1B / 16; i += 256)
      reinterpret_cast<uint4 *>(w1s)[i] = reinterpret_cast<const uint4 *>(a.w1c_frag_h)[i];
    for (int i = threadIdx.x; i < S::W2B / 16; i += 256)
      reinterpret_cast<uint4 *>(w2s)[i] = reinterpret_cast<const uint4 *>(a.w2_frag_h)[i];
    __syncthreads();
  }

  const int c = lane & 31, h = lane >> 5;
  const int r16 = lane & 15, g = lane >> 4;
  const int64_t n_tiles = (a.N + 31) >> 5;
  const int64_t n_qch = (a.B + MOL_QCHUNK - 1) / MOL_QCHUNK;
  const int64_t ntasks = n_tiles * n_qch;
  const int64_t wave = (int64_t)blockIdx.x * 4 + wv;
  const int64_t nwaves = (int64_t)gridDim.x * 4;

  // b2 in the accumulator layout of layer 2: component 32 pt + 8 (j / 4) + 4 h + j % 4
  f32x16 b2v[PT];
#pragma unroll
  for (int pt = 0; pt < PT; ++pt)
#pragma unroll
    for (int j = 0; j < 16; ++j) b2v[pt][j] = a.b2[32 * pt + 8 * (j >> 2) + 4 * h + (j & 3)];
  const uint4 ones = make_uint4(h == 0 ? 0x3C003C00u : 0u, 0u, 0u, 0u);  // k-slots 0 and 1 of the extra k-step: 1.0

  for (int64_t task = wave; task < ntasks; task += nwaves) {
    const int64_t tile = task / n_qch;
    const int b_lo = (int)(task % n_qch) * MOL_QCHUNK;
    const int b_hi = b_lo + MOL_QCHUNK < a.B ? b_lo + MOL_QCHUNK : a.B;
    const int64_t cpos = tile * 32 + c;
    const bool ok = cpos < a.N;
    const int64_t item = ok ? cpos : 0;

    // the item block: rows in MFMA operand order, and the cached gate halves decoded to fp32 in the layer-1
    // accumulator layout (hidden unit 32 mt + 8 q + 4 h + i at [mt][4 q + i])
    uint4 A[RT][SA];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      int64_t n = tile * 32 + rt * CPR + r16 / K_X;
      if (n >= a.N) n = 0;
      const char *rowp = a.embs + ((n * K_X + (r16 % K_X)) * D_P + 8 * g) * 2;
#pragma unroll
      for (int s = 0; s < SA; ++s) A[rt][s] = ld16(rowp + 64 * s);
    }
    f32x16 xif[MT];
    {
      const char *xp = a.xi + ((size_t)item * H + 4 * h) * 2;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const uint2 x = *reinterpret_cast<const uint2 *>(xp + (32 * mt + 8 * q) * 2);
          xif[mt][4 * q + 0] = dec16<F16>(x.x & 0xffffu);
          xif[mt][4 * q + 1] = dec16<F16>(x.x >> 16);
          xif[mt][4 * q + 2] = dec16<F16>(x.y & 0xffffu);
          xif[mt][4 * q + 3] = dec16<F16>(x.y >> 16);
        }
    }

    for (int b0 = b_lo; b0 < b_hi; b0 += QPM) {
      // ---- A: component logits of QPM queries -> LDS tiles (column r16 = (query b0 + r16 / K_U, ku = r16 % K_U)) ----
      // U of the group's queries, in operand form: issued first, needed only after the logits
      uint32_t upk[QPM][MT];
#pragma unroll
      for (int qi = 0; qi < QPM; ++qi) {
        const int bc = b0 + qi < b_hi ? b0 + qi : b_hi - 1;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) upk[qi][mt] = a.UP[((size_t)bc * MT + mt) * 64 + lane];
      }
      float res[QPM];
      uint4 Ff[SA];
      const bool qvalid = b0 * K_U + r16 < b_hi * K_U;
#pragma unroll
      for (int s = 0; s < SA; ++s)
        Ff[s] = qvalid ? ld16(a.F + ((size_t)(b0 * K_U + r16) * D_P + 32 * s + 8 * g) * 2) : make_uint4(0, 0, 0, 0);
      float *clw = cl + (r16 / K_U) * (32 * CLS) + (r16 % K_U) * K_X;
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < SA; ++s) acc = mfma16_16x16x32<F16>(A[rt][s], Ff[s], acc);
        // acc[j]: row 4 g + j of the tile = (candidate rt * CPR + (4 g + j) / K_X, kx (4 g + j) % K_X)
        if constexpr (K_X % 4 == 0) {
          float4 v = make_float4(acc[0] * a.logit_scale, acc[1] * a.logit_scale, acc[2] * a.logit_scale,
                                 acc[3] * a.logit_scale);
          *reinterpret_cast<float4 *>(&clw[(rt * CPR + (4 * g) / K_X) * CLS + (4 * g) % K_X]) = v;
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            clw[(rt * CPR + (4 * g + j) / K_X) * CLS + (4 * g + j) % K_X] = acc[j] * a.logit_scale;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

      // The QPM queries of the group are independent chains of dependent steps (LDS read -> MFMA -> convert -> MFMA ->
      // softmax): unrolled into one block with no branches so that the scheduler can overlap them.  A query past the
      // end of the chunk (incomplete last group) is computed on zero logits and not stored.
#pragma unroll
      for (int qi = 0; qi < QPM; ++qi) {
        const float *clq = cl + qi * (32 * CLS);
        // ---- B: layer 1 (transposed), accumulators start at the cached item half; one more k-step adds U[b] ----
        f32x16 acc1[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc1[mt] = xif[mt];
#pragma unroll
        for (int s = 0; s < S1; ++s) {
          const float4 lo = *reinterpret_cast<const float4 *>(&clq[c * CLS + 16 * s + 8 * h]);
          const float4 hi = *reinterpret_cast<const float4 *>(&clq[c * CLS + 16 * s + 8 * h + 4]);
          const uint4 bf = make_uint4(pack16x2<true>(lo.x, lo.y), pack16x2<true>(lo.z, lo.w), pack16x2<true>(hi.x, hi.y),
                                      pack16x2<true>(hi.z, hi.w));
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            uint4 af;
            if constexpr (WREG) af = w1r[mt * S1 + s];
            else af = *reinterpret_cast<const uint4 *>(w1s + ((mt * S1 + s) * 64 + lane) * 16);
            acc1[mt] = mfma16_32x32x16<true>(af, bf, acc1[mt]);
          }
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc1[mt] = mfma16_32x32x16<true>(make_uint4(upk[qi][mt], 0u, 0u, 0u), ones, acc1[mt]);

        // ---- C: ReLU on packed halves, layer 2 (transposed), accumulators start at b2 ----
        f32x16 acc2[PT];
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) acc2[pt] = b2v[pt];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
          for (int qq = 0; qq < 2; ++qq) {
            uint4 bf;
            uint32_t *bw = reinterpret_cast<uint32_t *>(&bf);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              f32x2v v = {acc1[mt][8 * qq + 2 * e], acc1[mt][8 * qq + 2 * e + 1]};
              f16x2v hv = __builtin_convertvector(v, f16x2v);
              const f16x2v zero = {(_Float16)0.f, (_Float16)0.f};
              hv = __builtin_elementwise_max(hv, zero);
              bw[e] = __builtin_bit_cast(uint32_t, hv);
            }
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
              uint4 af;
              if constexpr (WREG) af = w2r[pt * S2 + mt * 2 + qq];
              else af = *reinterpret_cast<const uint4 *>(w2s + ((pt * S2 + mt * 2 + qq) * 64 + lane) * 16);
              acc2[pt] = mfma16_32x32x16<true>(af, bf, acc2[pt]);
            }
          }
        }

        // ---- D: softmax over the components (base-2 exponentials) and the weighted sum ----
        float m = -INFINITY;
#pragma unroll
        for (int pt = 0; pt < PT; ++pt)
#pragma unroll
          for (int j = 0; j < 16; ++j)
            if (32 * pt + 8 * (j >> 2) < P) m = fmaxf(m, acc2[pt][j]);
        m = half_swap_max(m);
        constexpr float L2E = 1.4426950408889634f;
        const float mm = m * L2E;
        float den = 0.f, num = 0.f;
#pragma unroll
        for (int pt = 0; pt < PT; ++pt)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            if (32 * pt + 8 * q < P) {
              const float4 c4 = *reinterpret_cast<const float4 *>(&clq[c * CLS + 32 * pt + 8 * q + 4 * h]);
              const float e0 = __builtin_amdgcn_exp2f(fmaf(acc2[pt][4 * q + 0], L2E, -mm)),
                          e1 = __builtin_amdgcn_exp2f(fmaf(acc2[pt][4 * q + 1], L2E, -mm)),
                          e2 = __builtin_amdgcn_exp2f(fmaf(acc2[pt][4 * q + 2], L2E, -mm)),
                          e3 = __builtin_amdgcn_exp2f(fmaf(acc2[pt][4 * q + 3], L2E, -mm));
              den += (e0 + e1) + (e2 + e3);
              num += (e0 * c4.x + e1 * c4.y) + (e2 * c4.z + e3 * c4.w);
            }
          }
        den = half_swap_sum(den);
        num = half_swap_sum(num);
        res[qi] = num * __builtin_amdgcn_rcpf(den);
      }
      if (h == 0 && ok) {
#pragma unroll
        for (int qi = 0; qi < QPM; ++qi)
          if (b0 + qi < b_hi) a.scores[(size_t)(b0 + qi) * a.Kp + cpos] = res[qi];
      }
      // the next group overwrites the LDS logit tiles: all lanes must be done reading them
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// U[b, h] = sum_j W1u[h, j] * gu[b, j]: the user part of gating layer 1, once per query (Section 3.2).
// Eight lanes per output, 8 bf16 of each operand per load when the rows allow it; the partial sums meet in a fixed tree.
// UP (optional): the same value as a half head and half remainder, head | remainder << 16, laid out [B][H/32][64] with
// U[b, 32 mt + l] at [b][mt][l] and zeros at l >= 32 (exhaustive fast path).
__device__ __forceinline__ uint32_t half_head_and_rest(float v) {
  const _Float16 hd = (_Float16)v;
  const _Float16 rs = (_Float16)(v - (float)hd);
  return (uint32_t)__builtin_bit_cast(uint16_t, hd) | ((uint32_t)__builtin_bit_cast(uint16_t, rs) << 16);
}

#define USER_GATE_LPO 8  // lanes per output
__global__ void k_user_gate(const uint16_t *w1u, const uint16_t *gu, float *U, uint32_t *UP, int B, int H, int d_gu,
                            bool f16) {
  constexpr int LPO = USER_GATE_LPO;
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  int i = t / LPO;
  const int sub = t % LPO;
  const bool live = i < B * H;
  if (!live) i = B * H - 1;  // the lane still takes part in the exchange below
  const int b = i / H, hh = i % H;
  float acc = 0.f;
  if (d_gu % 8 != 0) {  // rows are not 16-byte aligned: element by element
    for (int j = sub; j < d_gu; j += LPO)
      acc = fmaf(dec16(w1u[(size_t)hh * d_gu + j], f16), dec16(gu[(size_t)b * d_gu + j], f16), acc);
  } else {
    // the LPO lanes of an output read consecutive 16-byte pieces of both rows (whole lines), four in flight per lane
    const uint4 *wr = reinterpret_cast<const uint4 *>(w1u + (size_t)hh * d_gu);
    const uint4 *gr = reinterpret_cast<const uint4 *>(gu + (size_t)b * d_gu);
    constexpr int PF = 4;
    const int np = d_gu / 8;
    for (int j0 = sub; j0 < np; j0 += LPO * PF) {
      uint4 wq[PF], gq[PF];
#pragma unroll
      for (int u = 0; u < PF; ++u) {
        const int j = j0 + u * LPO < np ? j0 + u * LPO : j0;
        wq[u] = wr[j];
        gq[u] = gr[j];
      }
#pragma unroll
      for (int u = 0; u < PF; ++u) {
        if (j0 + u * LPO >= np) break;
        const uint32_t wv[4] = {wq[u].x, wq[u].y, wq[u].z, wq[u].w}, gv[4] = {gq[u].x, gq[u].y, gq[u].z, gq[u].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc = fmaf(dec16(wv[e] & 0xffffu, f16), dec16(gv[e] & 0xffffu, f16), acc);
          acc = fmaf(dec16(wv[e] >> 16, f16), dec16(gv[e] >> 16, f16), acc);
        }
      }
    }
  }
#pragma unroll
  for (int o = 1; o < LPO; o <<= 1) acc += __shfl_xor(acc, o);
  if (live && sub == 0) {
    U[i] = acc;
    if (UP) {
      UP[((size_t)b * (H / 32) + hh / 32) * 64 + (hh & 31)] = half_head_and_rest(acc);
      UP[((size_t)b * (H / 32) + hh / 32) * 64 + 32 + (hh & 31)] = 0u;
    }
  }
}

// Decomposed gate, per query (userWeightFn of Algorithm 1): UW[b, :] = Wu2 * act(Wu1 * gu[b] + bu1) + bu2, and the
// bias of the cross MLP's first layer broadcast into U[b, :] (the scoring kernel adds U[b] to layer 1).
// One workgroup per query; the hidden units pass through LDS.
__global__ __launch_bounds__(256) void k_user_weights(const uint16_t *wu1, const float *bu1, const uint16_t *wu2,
                                                      const float *bu2, const float *b1c, const uint16_t *gu, float *UW,
                                                      float *U, int P, int H, int d_gu, int d_hu, int act, bool f16) {
  __shared__ float hid[1024];
  const int b = blockIdx.x;
  for (int i = threadIdx.x; i < d_hu; i += 256) {
    float acc = bu1[i];
    for (int j = 0; j < d_gu; ++j)
      acc = fmaf(dec16(wu1[(size_t)i * d_gu + j], f16), dec16(gu[(size_t)b * d_gu + j], f16), acc);
    hid[i] = act_fn(acc, act);
  }
  __syncthreads();
  for (int p = threadIdx.x; p < P; p += 256) {
    float acc = bu2[p];
    for (int i = 0; i < d_hu; ++i) acc = fmaf(dec16(wu2[(size_t)p * d_hu + i], f16), hid[i], acc);
    UW[(size_t)b * P + p] = acc;
  }
  for (int h = threadIdx.x; h < H; h += 256) U[(size_t)b * H + h] = b1c[h];
}

template <int K_U, int K_X, int D_P, int H, bool EXH, int FORM, bool F16, int K_G = 0, int D_S = 32, int D_HG = 64>
mol_status_t launch_shape(const MolArgs &a, hipStream_t st) {
  using S = MolShape<K_U, K_X, D_P, H>;
  using GS = GenShape<K_G, D_P, D_S, D_HG>;
  constexpr int NW = K_G ? 8 : 4;  // wavefronts per workgroup, as in the kernel
  constexpr size_t LDS = S::W1B + S::W2B + GS::LDS + S::PT * 32 * 4 + (size_t)NW * S::WAVE_FLOATS * 4;
  auto kern = k_mol_score<K_U, K_X, D_P, H, EXH, FORM, F16, K_G, D_S, D_HG>;
  // launch shape of this instantiation, found once per process (one GPU; concurrent first calls are serialised)
  static std::mutex mu;
  static bool configured = false;
  static int per_sm = 1, sm_count = 0;
  {
    std::lock_guard<std::mutex> lk(mu);
    if (!configured) {
      int dev = 0;
      HIP_TRY(hipGetDevice(&dev));
      HIP_TRY(hipDeviceGetAttribute(&sm_count, hipDeviceAttributeMultiprocessorCount, dev));
      HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)LDS));
      HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_sm, kern, NW * 64, LDS));
      if (per_sm < 1) per_sm = 1;
      configured = true;
    }
  }
  const int64_t ntiles = EXH ? ((a.Kp + 31) / 32) * ((a.B + MOL_QCHUNK - 1) / MOL_QCHUNK) : ((a.Kp + 31) / 32) * a.B;
  int64_t grid = (int64_t)sm_count * per_sm;
  const int64_t need = (ntiles + NW - 1) / NW;
  if (grid > need) grid = need;
  if (grid < 1) grid = 1;
  ProfScope ps(MOL_PROF_MOL_SCORE, st);
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NW * 64), LDS, st, a);
  HIP_TRY(hipGetLastError());
  return MOL_OK;
}

// launch of the exhaustive fast form
template <int K_U, int K_X, int D_P, int H, bool F16>
mol_status_t launch_exh(const MolArgs &a, hipStream_t st) {
  using S = MolShape<K_U, K_X, D_P, H>;
  constexpr int QPM = 16 / K_U;
  constexpr bool WREG = S::MT * S::S1 + S::PT * S::S2 <= 8;  // as in the kernel: weight fragments in registers
  constexpr size_t LDS = (WREG ? 0 : S::W1B + S::W2B) + (size_t)4 * QPM * 32 * S::CLS * 4;
  auto kern = k_mol_exh<K_U, K_X, D_P, H, F16>;
  static std::mutex mu;
  static bool configured = false;
  static int per_sm = 1, sm_count = 0;
  {
    std::lock_guard<std::mutex> lk(mu);
    if (!configured) {
      int dev = 0;
      HIP_TRY(hipGetDevice(&dev));
      HIP_TRY(hipDeviceGetAttribute(&sm_count, hipDeviceAttributeMultiprocessorCount, dev));
      HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS));
      HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_sm, kern, 256, LDS));
      if (per_sm < 1) per_sm = 1;
      configured = true;
    }
  }
  const int64_t ntasks = ((a.N + 31) / 32) * ((a.B + MOL_QCHUNK - 1) / MOL_QCHUNK);
  int64_t grid = (int64_t)sm_count * per_sm;
  const int64_t need = (ntasks + 3) / 4;
  if (grid > need) grid = need;
  if (grid < 1) grid = 1;
  ProfScope ps(MOL_PROF_MOL_SCORE, st);
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), LDS, st, a);
  HIP_TRY(hipGetLastError());
  return MOL_OK;
}

}  // namespace

mol_status_t launch_user_gate(const mol_corpus *c, const void *user_gate, int B, float *U, float *UW, uint32_t *UP,
                              hipStream_t st) {
  const int n = B * c->H;
  ProfScope ps(MOL_PROF_USER_GATE, st);
  if (c->gate_form == MOL_GATE_DECOMPOSED) {
    hipLaunchKernelGGL(k_user_weights, dim3(B), dim3(256), 0, st, static_cast<const uint16_t *>(c->wu1), c->bu1,
                       static_cast<const uint16_t *>(c->wu2), c->bu2, c->b1c, static_cast<const uint16_t *>(user_gate), UW,
                       U, c->P, c->H, c->d_gu, c->d_hu, c->act, c->f16);
    HIP_TRY(hipGetLastError());
    return MOL_OK;
  }
  hipLaunchKernelGGL(k_user_gate, dim3((n * USER_GATE_LPO + 255) / 256), dim3(256), 0, st, static_cast<const uint16_t *>(c->w1u),
                     static_cast<const uint16_t *>(user_gate), U, UP, B, c->H, c->d_gu, c->f16);
  HIP_TRY(hipGetLastError());
  return MOL_OK;
}

bool mol_shape_supported(int k_u, int k_x, int d_p, int H);

// shapes the exhaustive fast form is built for: those whose 32-item tile fits the register file (k_x <= 4)
#define MOL_EXH_SHAPES(X) \
  X(4, 4, 32, 32)         \
  X(4, 4, 64, 64)         \
  X(8, 4, 64, 128)        \
  X(16, 1, 32, 32)        \
  X(8, 2, 128, 96)

// (k_u, k_x, d_p, H, k_x_gen, d_s, d_hg) the kernel with generated item embeddings is built for (concatenated gate only)
#define MOL_GEN_SHAPES(X)     \
  X(4, 4, 64, 64, 2, 32, 64)  \
  X(8, 8, 64, 128, 2, 32, 64)

bool mol_gen_shape_supported(int k_u, int k_x, int d_p, int H, int k_g, int d_s, int d_hg) {
#define X(KU, KX, DP, HH, KG, DS, DHG) \
  if (k_u == KU && k_x == KX && d_p == DP && H == HH && k_g == KG && d_s == DS && d_hg == DHG) return true;
  MOL_GEN_SHAPES(X)
#undef X
  return false;
}

bool mol_exh_fast_form(const mol_corpus *c) {
  if (c->k_g > 0) return false;
  if (c->gate_form != MOL_GATE_CONCAT || c->act != MOL_ACT_RELU || !c->w1c_frag_h || !c->w2_frag_h) return false;
#define X(KU, KX, DP, HH) \
  if (c->k_u == KU && c->k_x == KX && c->d_p == DP && c->H == HH) return true;
  MOL_EXH_SHAPES(X)
#undef X
  return false;
}

#define MOL_SHAPES(X) \
  X(4, 4, 32, 32)     \
  X(4, 4, 64, 64)     \
  X(8, 4, 64, 128)    \
  X(8, 8, 64, 128)    \
  X(2, 8, 32, 64)     \
  X(16, 1, 32, 32)    \
  X(8, 2, 128, 96)

bool mol_shape_supported(int k_u, int k_x, int d_p, int H) {
#define X(KU, KX, DP, HH) \
  if (k_u == KU && k_x == KX && d_p == DP && H == HH) return true;
  MOL_SHAPES(X)
#undef X
  return false;
}

// Index select (Section 4.1.3): out[b, c, :] = item row cand[b, c] (row_bytes = k_x * d_p * 2, a multiple of 64), zeros
// for padding.  Consecutive lanes copy consecutive 16-byte pieces of a row, so every request covers whole cache lines
// of one row; a wavefront handles rows_per_wave rows per instruction.
__global__ __launch_bounds__(256) void k_gather_items(const char *embs, const int32_t *cand, int64_t npairs, int64_t N,
                                                      int row_bytes, char *out) {
  const int pieces = row_bytes / 16;                    // 16-byte pieces per row (4 .. 128)
  const int64_t total = npairs * pieces;
  const int64_t stride = (int64_t)gridDim.x * 256 * 4;
  for (int64_t base = ((int64_t)blockIdx.x * 256 + threadIdx.x); base < total; base += stride) {
    uint4 v[4];
    int64_t at[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      at[u] = base + (int64_t)u * gridDim.x * 256;
      v[u] = make_uint4(0, 0, 0, 0);
      if (at[u] < total) {
        const int64_t pair = at[u] / pieces;
        const int piece = (int)(at[u] % pieces);
        const int32_t id = cand[pair];
        if (id >= 0 && id < N) v[u] = ld16(embs + (size_t)id * row_bytes + (size_t)piece * 16);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (at[u] < total) *reinterpret_cast<uint4 *>(out + (size_t)at[u] * 16) = v[u];
  }
}

mol_status_t launch_gather_items(const mol_corpus *c, const int32_t *cand_idx, int B, int64_t Kp, void *out, hipStream_t st) {
  const int row_bytes = (c->k_x - c->k_g) * c->d_p * 2;  // the cached embeddings of an item
  const int64_t npairs = (int64_t)B * Kp;
  const int64_t total = npairs * (row_bytes / 16);
  int64_t grid = (total + 1023) / 1024;
  if (grid > 256 * 16) grid = 256 * 16;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL(k_gather_items, dim3((unsigned)grid), dim3(256), 0, st, static_cast<const char *>(c->embs), cand_idx,
                     npairs, c->N, row_bytes, static_cast<char *>(out));
  HIP_TRY(hipGetLastError());
  return MOL_OK;
}

template <int K_U, int K_X, int D_P, int H>
static mol_status_t launch_variant(const MolArgs &a, bool exhaustive, int form, bool f16, hipStream_t st) {
#define V(E, F, T) launch_shape<K_U, K_X, D_P, H, E, F, T>(a, st)
  if (f16) {
    if (form == 0) return exhaustive ? V(true, 0, true) : V(false, 0, true);
    return exhaustive ? V(true, 1, true) : V(false, 1, true);
  }
  if (form == 0) return exhaustive ? V(true, 0, false) : V(false, 0, false);
  return exhaustive ? V(true, 1, false) : V(false, 1, false);
#undef V
}

mol_status_t launch_mol_score(const mol_corpus *c, const void *user_embs, const float *U, const float *UW,
                              const uint32_t *UP, int B, const int32_t *cand_idx, const int32_t *cand_count, int64_t Kp,
                              float *scores, hipStream_t st) {
  MolArgs a;
  a.embs = static_cast<const char *>(c->embs);
  a.xi = static_cast<const char *>(c->xi);
  a.w1c_frag = static_cast<const char *>(c->w1c_frag);
  a.w2_frag = static_cast<const char *>(c->w2_frag);
  a.b2 = c->b2;
  a.F = static_cast<const char *>(user_embs);
  a.U = U;
  a.xw = c->xw;
  a.UW = UW;
  a.cand = cand_idx;
  a.cand_count = cand_idx ? cand_count : nullptr;
  a.scores = scores;
  a.Kp = cand_idx ? Kp : c->N;
  a.N = c->N;
  a.B = B;
  a.act = c->act;
  a.logit_scale = c->logit_scale;
  a.w1c_frag_h = static_cast<const char *>(c->w1c_frag_h);
  a.w2_frag_h = static_cast<const char *>(c->w2_frag_h);
  a.UP = UP;
  a.seed = static_cast<const char *>(c->seed);
  a.wg1_frag = static_cast<const char *>(c->wg1_frag);
  a.wg2_frag = static_cast<const char *>(c->wg2_frag);
  a.bg1 = c->bg1;
  a.bg2 = c->bg2;
  if (c->k_g > 0) {  // generated item embeddings: the per-candidate form also serves cand_idx = NULL (candidate c = item c)
#define XG(KU, KX, DP, HH, KG, DS, DHG)                                                                               \
  if (c->k_u == KU && c->k_x == KX && c->d_p == DP && c->H == HH && c->k_g == KG && c->d_s == DS && c->d_hg == DHG)   \
    return c->f16 ? launch_shape<KU, KX, DP, HH, false, 0, true, KG, DS, DHG>(a, st)                                  \
                  : launch_shape<KU, KX, DP, HH, false, 0, false, KG, DS, DHG>(a, st);
    MOL_GEN_SHAPES(XG)
#undef XG
    return mol_fail(MOL_EUNSUPPORTED, "no generator instance for this shape");
  }
  if (mol_exh_fast_form(c) && cand_idx == nullptr && UP != nullptr) {
#define XF(KU, KX, DP, HH)                                                \
  if (c->k_u == KU && c->k_x == KX && c->d_p == DP && c->H == HH)         \
    return c->f16 ? launch_exh<KU, KX, DP, HH, true>(a, st) : launch_exh<KU, KX, DP, HH, false>(a, st);
    MOL_EXH_SHAPES(XF)
#undef XF
  }
#define X(KU, KX, DP, HH) \
  if (c->k_u == KU && c->k_x == KX && c->d_p == DP && c->H == HH) return launch_variant<KU, KX, DP, HH>(a, cand_idx == nullptr, c->gate_form, c->f16, st);
  MOL_SHAPES(X)
#undef X
  return mol_fail(MOL_EUNSUPPORTED, "no MoL kernel built for k_u=%d k_x=%d d_p=%d H=%d", c->k_u, c->k_x, c->d_p, c->H);
}
