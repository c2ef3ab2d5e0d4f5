// mol_corpus_pack: the item-side cache (Section 2.2; the loops marked cachable in Algorithm 1).
//   * gating weights re-laid into the matrix-core fragment order the scoring kernel reads from LDS,
//   * Xi[n, :] = W1x * item_gate[n] + b1 for every item, bf16 (the cached "item-side gating weights").
#include <math.h>
#include <stdlib.h>

#include "common.hpp"

bool mol_shape_supported(int k_u, int k_x, int d_p, int H);

namespace {

// One thread per output element of the fragment buffers and the small copies.
__global__ void k_pack_weights(const uint16_t *W1, const uint16_t *W2, const float *b2, int P, int H, int d_gu,
                               int d_gx, uint16_t *w1c_frag, uint16_t *w2_frag, uint16_t *w1u, uint16_t *w1x,
                               float *b2p) {
  const int d_in = P + d_gu + d_gx;
  const int MT = H / 32, S1 = P / 16, PT = (P + 31) / 32, S2 = H / 16;
  const int n1 = MT * S1 * 512, n2 = PT * S2 * 512, n3 = H * d_gu, n4 = H * d_gx, n5 = PT * 32;
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n1) {
    // layer-1 cross part, A operand of a 32x32x16 product: lane l holds row l%32, k = 8*(l/32) + e
    const int e = i & 7, l = (i >> 3) & 63, f = i >> 9;
    const int mt = f / S1, s = f % S1;
    w1c_frag[i] = W1[(size_t)(32 * mt + (l & 31)) * d_in + 16 * s + 8 * (l >> 5) + e];
    return;
  }
  i -= n1;
  if (i < n2) {
    // layer-2 weights; k-slot (half, e) of k-step (mt, qq) is hidden unit 32mt + 16qq + 8*(e/4) + 4*half + e%4,
    // which is where the layer-1 accumulators of the scoring kernel hold that unit
    const int e = i & 7, l = (i >> 3) & 63, f = i >> 9;
    const int pt = f / S2, s2 = f % S2;
    const int mt = s2 >> 1, qq = s2 & 1;
    const int p = 32 * pt + (l & 31);
    const int hu = 32 * mt + 16 * qq + 8 * (e >> 2) + 4 * (l >> 5) + (e & 3);
    w2_frag[i] = (p < P) ? W2[(size_t)p * H + hu] : (uint16_t)0;
    return;
  }
  i -= n2;
  if (i < n3) {
    w1u[i] = W1[(size_t)(i / d_gu) * d_in + P + (i % d_gu)];
    return;
  }
  i -= n3;
  if (i < n4) {
    w1x[i] = W1[(size_t)(i / d_gx) * d_in + P + d_gu + (i % d_gx)];
    return;
  }
  i -= n4;
  if (i < n5) b2p[i] = (b2 && i < P) ? b2[i] : 0.f;
}

// bf16 -> IEEE half, element by element (exact for normal halves: 8 significant bits fit 11; magnitudes below 2^-14 land
// on the half subnormal grid, absolute error <= 2^-25).  For the fragment buffers of the exhaustive fast form.
__global__ void k_bf16_to_f16(const uint16_t *src, uint16_t *dst, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = __builtin_bit_cast(uint16_t, (_Float16)bf16_bits_to_f32(src[i]));
}

// 16-bit (bf16 or half) -> IEEE half over a large tensor (the seed table of generated item embeddings).
__global__ void k_to_f16_big(const uint16_t *src, uint16_t *dst, int64_t n, bool src_f16) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = src_f16 ? src[i] : __builtin_bit_cast(uint16_t, (_Float16)bf16_bits_to_f32(src[i]));
}

// Generator weights (Section 3.1, on-the-fly item embeddings) as the row operands of 16x16x32 half MFMAs: lane l holds row
// l % 16 of a 16-row tile and the 8 k values of group l / 16.
//   layer 1, tile ut, k-step s : Wg1[16 ut + l % 16][32 s + 8 (l / 16) + e]
//   layer 2, tile ft, k-step s : Wg2[16 ft + l % 16][u(e)],  u(e) = 32 s + 4 (l / 16) + e for e < 4,
//                                                                   32 s + 16 + 4 (l / 16) + (e - 4) otherwise
// (the hidden units reach layer 2 as two 16-row result tiles side by side: lane group g holds rows 4 g .. 4 g + 3 of each).
__global__ void k_pack_gen_weights(const uint16_t *Wg1, const uint16_t *Wg2, int d_s, int d_hg, int n_out, bool src_f16,
                                   uint16_t *wg1_frag, uint16_t *wg2_frag) {
  const int SG1 = d_s / 32, SG2 = d_hg / 32;
  const int n1 = (d_hg / 16) * SG1 * 512, n2 = (n_out / 16) * SG2 * 512;
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  auto cv = [&](uint16_t v) -> uint16_t { return src_f16 ? v : __builtin_bit_cast(uint16_t, (_Float16)bf16_bits_to_f32(v)); };
  if (i < n1) {
    const int e = i & 7, l = (i >> 3) & 63, f = i >> 9;
    const int ut = f / SG1, s = f % SG1;
    wg1_frag[i] = cv(Wg1[(size_t)(16 * ut + (l & 15)) * d_s + 32 * s + 8 * (l >> 4) + e]);
    return;
  }
  i -= n1;
  if (i < n2) {
    const int e = i & 7, l = (i >> 3) & 63, f = i >> 9;
    const int ft = f / SG2, s = f % SG2, g = l >> 4;
    const int u = e < 4 ? 32 * s + 4 * g + e : 32 * s + 16 + 4 * g + (e - 4);
    wg2_frag[i] = cv(Wg2[(size_t)(16 * ft + (l & 15)) * d_hg + u]);
  }
}

// Xi^T[h, n] = W1x[h, :] . gx[n, :] + b1[h] on 32x32x16 MFMA: A = W1x rows (hidden units), B = item rows.
// A wavefront takes 32 items; lane (c = lane%32, half) loads its item's row chunks once and walks the hidden tiles.
template <int KS, bool F16>  // d_gx / 16; 16-bit type of the inputs and of Xi
__global__ __launch_bounds__(256) void k_item_gate_cache(const char *gx, const char *w1x, const float *b1,
                                                         uint16_t *xi, int64_t N, int H) {
  const int lane = threadIdx.x & 63;
  const int c = lane & 31, h = lane >> 5;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  const int64_t ntiles = (N + 31) >> 5;
  constexpr int DG = KS * 16;
  for (int64_t tile = wave; tile < ntiles; tile += nwaves) {
    int64_t n = tile * 32 + c;
    const bool ok = n < N;
    if (!ok) n = N - 1;
    uint4 bfrag[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) bfrag[s] = ld16(gx + ((size_t)n * DG + 16 * s + 8 * h) * 2);
    for (int mt = 0; mt < H / 32; ++mt) {
      f32x16 acc;
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[j] = 0.f;
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const uint4 af = ld16(w1x + ((size_t)(32 * mt + c) * DG + 16 * s + 8 * h) * 2);
        acc = mfma16_32x32x16<F16>(af, bfrag[s], acc);
      }
      mfma_settle();
      if (ok) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int hu = 32 * mt + 8 * q + 4 * h;
          float v[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = acc[4 * q + i] + (b1 ? b1[hu + i] : 0.f);
          uint2 o = make_uint2(pack16x2<F16>(v[0], v[1]), pack16x2<F16>(v[2], v[3]));
          *reinterpret_cast<uint2 *>(xi + (size_t)n * H + hu) = o;
        }
      }
    }
  }
}

// Decomposed gate: xw[n, :] = Wx2 * act(Wx1 * gx[n] + bx1) + bx2 (itemWeightFn of Algorithm 1, the cachable item-side
// gating weights), f32 [N, P].  A workgroup takes 32 items at a time: features and hidden units live in LDS, a
// wavefront's lanes share a weight row and differ in the item, results leave through LDS in whole rows.
__global__ __launch_bounds__(256) void k_item_weights(const uint16_t *gx, const uint16_t *Wx1, const float *bx1,
                                                      const uint16_t *Wx2, const float *bx2, float *xw, int64_t N,
                                                      int d_gx, int d_hx, int P, int act, bool f16) {
  extern __shared__ float lds_iw[];
  const int sg = d_gx + 1, sh = d_hx + 1, sp = P + 1;
  float *gxs = lds_iw;               // [32][sg], reused as out [32][sp] (P <= 128, d_gx >= 16: see the launcher)
  float *hid = lds_iw + 32 * (sg > sp ? sg : sp);  // [32][sh]
  const int64_t nblk = (N + 31) / 32;
  for (int64_t blk = blockIdx.x; blk < nblk; blk += gridDim.x) {
    const int64_t n0 = blk * 32;
    const int cnt = (int)((N - n0) < 32 ? (N - n0) : 32);
    __syncthreads();
    for (int i = threadIdx.x; i < 32 * d_gx; i += 256) {
      const int it = i / d_gx, j = i % d_gx;
      gxs[it * sg + j] = it < cnt ? dec16(gx[(size_t)(n0 + it) * d_gx + j], f16) : 0.f;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 32 * d_hx; i += 256) {
      const int it = i & 31, u = i >> 5;
      float acc = bx1 ? bx1[u] : 0.f;
      const uint16_t *w = Wx1 + (size_t)u * d_gx;
      for (int j = 0; j < d_gx; ++j) acc = fmaf(dec16(w[j], f16), gxs[it * sg + j], acc);
      hid[it * sh + u] = act == MOL_ACT_RELU ? fmaxf(acc, 0.f) : acc / (1.f + __expf(-acc));
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 32 * P; i += 256) {
      const int it = i & 31, p = i >> 5;
      float acc = bx2 ? bx2[p] : 0.f;
      const uint16_t *w = Wx2 + (size_t)p * d_hx;
      for (int j = 0; j < d_hx; ++j) acc = fmaf(dec16(w[j], f16), hid[it * sh + j], acc);
      gxs[it * sp + p] = acc;  // the features are no longer needed
    }
    __syncthreads();
    for (int i = threadIdx.x; i < cnt * P; i += 256) xw[(size_t)n0 * P + i] = gxs[(i / P) * sp + (i % P)];
  }
}

}  // namespace

mol_status_t launch_item_weights(const mol_corpus *c, const mol_config_t *cfg, const void *item_gate, hipStream_t st) {
  int dev = 0, sms = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&sms, hipDeviceAttributeMultiprocessorCount, dev));
  const int sg = c->d_gx + 1, sh = cfg->d_hx + 1, sp = c->P + 1;
  const size_t lds = ((size_t)32 * (sg > sp ? sg : sp) + (size_t)32 * sh) * 4;
  if (lds > 160 * 1024) return mol_fail(MOL_EUNSUPPORTED, "d_hx=%d is too wide for the item-weight kernel", cfg->d_hx);
  if (lds > 48 * 1024)
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(k_item_weights), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  int64_t grid = (int64_t)sms * 8;
  const int64_t need = (c->N + 31) / 32;
  if (grid > need) grid = need;
  hipLaunchKernelGGL(k_item_weights, dim3((unsigned)grid), dim3(256), lds, st, static_cast<const uint16_t *>(item_gate),
                     static_cast<const uint16_t *>(cfg->Wx1), cfg->bx1, static_cast<const uint16_t *>(cfg->Wx2), cfg->bx2,
                     c->xw, c->N, c->d_gx, cfg->d_hx, c->P, c->act, c->f16);
  HIP_TRY(hipGetLastError());
  return MOL_OK;
}

mol_status_t launch_item_gate_cache(const mol_corpus *c, const void *item_gate, const void *w1x, const float *b1,
                                    hipStream_t st) {
  int dev = 0, sms = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&sms, hipDeviceAttributeMultiprocessorCount, dev));
  int64_t grid = (int64_t)sms * 4;
  const int64_t need = ((c->N + 31) / 32 + 3) / 4;
  if (grid > need) grid = need;
  if (grid < 1) grid = 1;
  const char *gx = static_cast<const char *>(item_gate);
  const char *w = static_cast<const char *>(w1x);
  uint16_t *xi = static_cast<uint16_t *>(c->xi);
#define LAUNCH(KS)                                                                                                      \
  if (c->f16)                                                                                                           \
    hipLaunchKernelGGL((k_item_gate_cache<KS, true>), dim3((unsigned)grid), dim3(256), 0, st, gx, w, b1, xi, c->N, c->H);  \
  else                                                                                                                  \
    hipLaunchKernelGGL((k_item_gate_cache<KS, false>), dim3((unsigned)grid), dim3(256), 0, st, gx, w, b1, xi, c->N, c->H); \
  break;
  switch (c->d_gx / 16) {
    case 1: LAUNCH(1)
    case 2: LAUNCH(2)
    case 4: LAUNCH(4)
    case 6: LAUNCH(6)
    case 8: LAUNCH(8)
    case 16: LAUNCH(16)
    default:
      return mol_fail(MOL_EUNSUPPORTED, "d_gx=%d: supported widths are 16, 32, 64, 96, 128, 256", c->d_gx);
  }
#undef LAUNCH
  HIP_TRY(hipGetLastError());
  return MOL_OK;
}

extern "C" mol_status_t mol_corpus_pack(const mol_config_t *cfg, const void *stage1_items, const void *item_embs,
                                        const void *item_gate, void *stream, mol_corpus_t **out) {
  if (!cfg || !out) return mol_fail(MOL_EINVAL, "mol_corpus_pack: cfg and out must not be NULL");
  if (!item_embs || !item_gate || !cfg->W1 || !cfg->W2)
    return mol_fail(MOL_EINVAL, "mol_corpus_pack: item_embs, item_gate, W1 and W2 must not be NULL");
  if (cfg->N < 1 || cfg->N >= (int64_t)1 << 31) return mol_fail(MOL_EINVAL, "N=%lld must be in [1, 2^31)", (long long)cfg->N);
  if (cfg->d1 != 0 && cfg->d1 != 64) return mol_fail(MOL_EUNSUPPORTED, "d1=%d: the stage-1 kernels are built for d1 = 64", cfg->d1);
  if (cfg->d1 != 0 && !stage1_items) return mol_fail(MOL_EINVAL, "stage1_items is NULL but d1 != 0");
  if (cfg->stage1_dtype != MOL_F32 && cfg->stage1_dtype != MOL_BF16 && cfg->stage1_dtype != MOL_INT8)
    return mol_fail(MOL_EINVAL, "bad stage1_dtype");
  if (cfg->act != MOL_ACT_RELU && cfg->act != MOL_ACT_SILU) return mol_fail(MOL_EINVAL, "bad act");
  if (!mol_shape_supported(cfg->k_u, cfg->k_x, cfg->d_p, cfg->H))
    return mol_fail(MOL_EUNSUPPORTED, "no MoL kernel built for k_u=%d k_x=%d d_p=%d H=%d", cfg->k_u, cfg->k_x,
                    cfg->d_p, cfg->H);
  if (cfg->d_gu < 1 || cfg->d_gu > 1024) return mol_fail(MOL_EINVAL, "d_gu=%d out of range", cfg->d_gu);
  switch (cfg->d_gx) {
    case 16: case 32: case 64: case 96: case 128: case 256: break;
    default: return mol_fail(MOL_EUNSUPPORTED, "d_gx=%d: supported widths are 16, 32, 64, 96, 128, 256", cfg->d_gx);
  }
  if (cfg->mol_dtype != 0 && cfg->mol_dtype != MOL_BF16 && cfg->mol_dtype != MOL_F16)
    return mol_fail(MOL_EINVAL, "mol_dtype must be 0, MOL_BF16 or MOL_F16");
  const bool decomposed = cfg->gate_form == MOL_GATE_DECOMPOSED;
  if (cfg->gate_form != MOL_GATE_CONCAT && !decomposed) return mol_fail(MOL_EINVAL, "bad gate_form");
  const int k_g = cfg->k_x_gen;
  if (k_g < 0) return mol_fail(MOL_EINVAL, "k_x_gen must be >= 0");
  if (k_g > 0) {
    if (!cfg->item_seed || !cfg->Wg1 || !cfg->Wg2) return mol_fail(MOL_EINVAL, "generated embeddings need item_seed, Wg1 and Wg2");
    if (decomposed) return mol_fail(MOL_EUNSUPPORTED, "generated embeddings are built for the concatenated gate only");
    if (!mol_gen_shape_supported(cfg->k_u, cfg->k_x, cfg->d_p, cfg->H, k_g, cfg->d_s, cfg->d_hg))
      return mol_fail(MOL_EUNSUPPORTED, "no kernel with generated embeddings for k_u=%d k_x=%d d_p=%d H=%d k_x_gen=%d d_s=%d d_hg=%d",
                      cfg->k_u, cfg->k_x, cfg->d_p, cfg->H, k_g, cfg->d_s, cfg->d_hg);
  }
  if (decomposed) {
    if (!cfg->Wu1 || !cfg->Wu2 || !cfg->Wx1 || !cfg->Wx2)
      return mol_fail(MOL_EINVAL, "the decomposed gate needs Wu1, Wu2, Wx1 and Wx2");
    if (cfg->d_hu < 16 || cfg->d_hu > 1024 || cfg->d_hx < 16 || cfg->d_hx > 1024)
      return mol_fail(MOL_EINVAL, "d_hu=%d, d_hx=%d must be in [16, 1024]", cfg->d_hu, cfg->d_hx);
  }
  hipStream_t st = static_cast<hipStream_t>(stream);

  mol_corpus *c = static_cast<mol_corpus *>(calloc(1, sizeof(mol_corpus)));
  if (!c) return mol_fail(MOL_ENOMEM, "host allocation failed");
  c->N = cfg->N;
  c->d1 = cfg->d1;
  c->stage1_dtype = cfg->stage1_dtype;
  c->k_u = cfg->k_u;
  c->k_x = cfg->k_x;
  c->d_p = cfg->d_p;
  c->P = cfg->k_u * cfg->k_x;
  c->d_gu = cfg->d_gu;
  c->d_gx = cfg->d_gx;
  c->H = cfg->H;
  c->act = cfg->act;
  c->logit_scale = cfg->logit_scale;
  c->flags = cfg->flags;
  c->gate_form = cfg->gate_form;
  c->f16 = cfg->mol_dtype == MOL_F16;
  c->d_hu = decomposed ? cfg->d_hu : 0;
  c->k_g = k_g;
  c->d_s = k_g ? cfg->d_s : 0;
  c->d_hg = k_g ? cfg->d_hg : 0;
  (void)hipGetDevice(&c->device);

  const int P = c->P, H = c->H;
  const int MT = H / 32, S1 = P / 16, PT = (P + 31) / 32, S2 = H / 16;
  // the first layer of the decomposed gate's cross MLP has the P logits as its only input: no user / item columns
  const int w1_gu = decomposed ? 0 : c->d_gu, w1_gx = decomposed ? 0 : c->d_gx;
  const size_t n1 = (size_t)MT * S1 * 512, n2 = (size_t)PT * S2 * 512, n3 = (size_t)H * w1_gu,
               n4 = (size_t)H * w1_gx, n5 = (size_t)PT * 32;
  void *w1x = nullptr;
  mol_status_t rc = MOL_OK;
#define ALLOC(ptr, bytes)                                                                                  \
  if (rc == MOL_OK && hipMalloc(reinterpret_cast<void **>(&(ptr)), (bytes)) != hipSuccess) {               \
    (void)hipGetLastError();                                                                               \
    rc = mol_fail(MOL_ENOMEM, "hipMalloc of %zu bytes failed (%s)", (size_t)(bytes), #ptr);               \
  }
  ALLOC(c->w1c_frag, n1 * 2)
  ALLOC(c->w2_frag, n2 * 2)
  ALLOC(c->w1u, (n3 ? n3 : 1) * 2)
  ALLOC(w1x, (n4 ? n4 : 1) * 2)
  ALLOC(c->b2, n5 * 4)
  if (!decomposed && !c->f16) {
    ALLOC(c->w1c_frag_h, n1 * 2)
    ALLOC(c->w2_frag_h, n2 * 2)
  }
  if (decomposed) {
    ALLOC(c->xw, (size_t)c->N * P * 4)
    ALLOC(c->wu1, (size_t)cfg->d_hu * c->d_gu * 2)
    ALLOC(c->wu2, (size_t)P * cfg->d_hu * 2)
    ALLOC(c->bu1, (size_t)cfg->d_hu * 4)
    ALLOC(c->bu2, (size_t)P * 4)
    ALLOC(c->b1c, (size_t)H * 4)
  } else {
    ALLOC(c->xi, (size_t)c->N * H * 2)
  }
  const size_t ng1 = k_g ? (size_t)(cfg->d_hg / 16) * (cfg->d_s / 32) * 512 : 0;
  const size_t ng2 = k_g ? (size_t)(k_g * cfg->d_p / 16) * (cfg->d_hg / 32) * 512 : 0;
  if (k_g) {
    ALLOC(c->seed, (size_t)c->N * cfg->d_s * 2)
    ALLOC(c->wg1_frag, ng1 * 2)
    ALLOC(c->wg2_frag, ng2 * 2)
    ALLOC(c->bg1, (size_t)cfg->d_hg * 4)
    ALLOC(c->bg2, (size_t)k_g * cfg->d_p * 4)
  }
  void *s1copy = nullptr, *embcopy = nullptr;
  const size_t s1_bytes = (size_t)c->N * c->d1 * (c->stage1_dtype == MOL_F32 ? 4 : (c->stage1_dtype == MOL_BF16 ? 2 : 1));
  const size_t emb_bytes = (size_t)c->N * (c->k_x - k_g) * c->d_p * 2;  // the cached embeddings
  if (c->d1 && !(cfg->flags & MOL_PACK_BORROW_STAGE1)) { ALLOC(s1copy, s1_bytes) }
  if (!(cfg->flags & MOL_PACK_BORROW_EMBS)) { ALLOC(embcopy, emb_bytes) }
#undef ALLOC
  if (rc == MOL_OK) {
    c->stage1 = s1copy ? s1copy : stage1_items;
    c->own_stage1 = s1copy != nullptr;
    c->embs = embcopy ? embcopy : item_embs;
    c->own_embs = embcopy != nullptr;
    hipError_t e = hipSuccess;
    if (s1copy) e = hipMemcpyAsync(s1copy, stage1_items, s1_bytes, hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess && embcopy) e = hipMemcpyAsync(embcopy, item_embs, emb_bytes, hipMemcpyDeviceToDevice, st);
    if (e != hipSuccess) rc = mol_fail(MOL_EHIP, "device copy failed: %s", hipGetErrorString(e));
  }
  if (rc == MOL_OK) {
    const size_t total = n1 + n2 + n3 + n4 + n5;
    hipLaunchKernelGGL(k_pack_weights, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       static_cast<const uint16_t *>(cfg->W1), static_cast<const uint16_t *>(cfg->W2), cfg->b2, P, H,
                       w1_gu, w1_gx, static_cast<uint16_t *>(c->w1c_frag), static_cast<uint16_t *>(c->w2_frag),
                       static_cast<uint16_t *>(c->w1u), static_cast<uint16_t *>(w1x), c->b2);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) rc = mol_fail(MOL_EHIP, "k_pack_weights: %s", hipGetErrorString(e));
  }
  if (rc == MOL_OK && !decomposed) {
    if (c->f16) {
      c->w1c_frag_h = c->w1c_frag;
      c->w2_frag_h = c->w2_frag;
    } else {
      hipLaunchKernelGGL(k_bf16_to_f16, dim3((unsigned)((n1 + 255) / 256)), dim3(256), 0, st,
                         static_cast<const uint16_t *>(c->w1c_frag), static_cast<uint16_t *>(c->w1c_frag_h), (int)n1);
      hipLaunchKernelGGL(k_bf16_to_f16, dim3((unsigned)((n2 + 255) / 256)), dim3(256), 0, st,
                         static_cast<const uint16_t *>(c->w2_frag), static_cast<uint16_t *>(c->w2_frag_h), (int)n2);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) rc = mol_fail(MOL_EHIP, "k_bf16_to_f16: %s", hipGetErrorString(e));
    }
  }
  if (rc == MOL_OK && !decomposed) rc = launch_item_gate_cache(c, item_gate, w1x, cfg->b1, st);
  if (rc == MOL_OK && decomposed) {
    auto copy_or_zero = [&](void *dst, const void *src, size_t bytes) -> hipError_t {
      return src ? hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, st) : hipMemsetAsync(dst, 0, bytes, st);
    };
    hipError_t e = copy_or_zero(c->wu1, cfg->Wu1, (size_t)cfg->d_hu * c->d_gu * 2);
    if (e == hipSuccess) e = copy_or_zero(c->wu2, cfg->Wu2, (size_t)P * cfg->d_hu * 2);
    if (e == hipSuccess) e = copy_or_zero(c->bu1, cfg->bu1, (size_t)cfg->d_hu * 4);
    if (e == hipSuccess) e = copy_or_zero(c->bu2, cfg->bu2, (size_t)P * 4);
    if (e == hipSuccess) e = copy_or_zero(c->b1c, cfg->b1, (size_t)H * 4);
    if (e != hipSuccess) rc = mol_fail(MOL_EHIP, "copy of the user-side gate weights failed: %s", hipGetErrorString(e));
    if (rc == MOL_OK) rc = launch_item_weights(c, cfg, item_gate, st);
  }
  if (rc == MOL_OK && k_g) {
    const int64_t ns = c->N * cfg->d_s;
    hipLaunchKernelGGL(k_to_f16_big, dim3((unsigned)((ns + 255) / 256 < 65536 ? (ns + 255) / 256 : 65536)), dim3(256), 0, st,
                       static_cast<const uint16_t *>(cfg->item_seed), static_cast<uint16_t *>(c->seed), ns, c->f16);
    hipLaunchKernelGGL(k_pack_gen_weights, dim3((unsigned)((ng1 + ng2 + 255) / 256)), dim3(256), 0, st,
                       static_cast<const uint16_t *>(cfg->Wg1), static_cast<const uint16_t *>(cfg->Wg2), cfg->d_s, cfg->d_hg,
                       k_g * cfg->d_p, c->f16, static_cast<uint16_t *>(c->wg1_frag), static_cast<uint16_t *>(c->wg2_frag));
    hipError_t e = hipGetLastError();
    auto copy_or_zero = [&](void *dst, const void *src, size_t bytes) -> hipError_t {
      return src ? hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, st) : hipMemsetAsync(dst, 0, bytes, st);
    };
    if (e == hipSuccess) e = copy_or_zero(c->bg1, cfg->bg1, (size_t)cfg->d_hg * 4);
    if (e == hipSuccess) e = copy_or_zero(c->bg2, cfg->bg2, (size_t)k_g * cfg->d_p * 4);
    if (e != hipSuccess) rc = mol_fail(MOL_EHIP, "packing the generator failed: %s", hipGetErrorString(e));
  }
  if (rc == MOL_OK) {
    hipError_t e = hipStreamSynchronize(st);
    if (e != hipSuccess) rc = mol_fail(MOL_EHIP, "pack kernels failed: %s", hipGetErrorString(e));
  }
  if (w1x) (void)hipFree(w1x);
  if (rc != MOL_OK) {
    c->stage1 = s1copy;
    c->own_stage1 = s1copy != nullptr;
    c->embs = embcopy;
    c->own_embs = embcopy != nullptr;
    mol_corpus_free(c);
    return rc;
  }
  *out = c;
  return MOL_OK;
}

// Symmetric INT8 quantisation of stage-1 vectors (Section 4.1.1): q = clamp(rint(x * scale), -127, 127); the product is
// taken in fp32 (one rounding), rint rounds halves to even.  8 elements per thread.
template <bool SRC_BF16>
__global__ void k_quantize_int8(const void *src, int64_t n, float scale, int8_t *dst) {
  const int64_t i0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 8;
  if (i0 >= n) return;
  float v[8];
  const int m = (n - i0) < 8 ? (int)(n - i0) : 8;
  if (m == 8) {
    if (SRC_BF16) {
      const uint4 u = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(src) + i0);
      const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[2 * e] = bf16_bits_to_f32(w[e] & 0xffffu);
        v[2 * e + 1] = bf16_bits_to_f32(w[e] >> 16);
      }
    } else {
      const float4 a = *reinterpret_cast<const float4 *>(static_cast<const float *>(src) + i0);
      const float4 b = *reinterpret_cast<const float4 *>(static_cast<const float *>(src) + i0 + 4);
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
      v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
  } else {
    for (int e = 0; e < m; ++e)
      v[e] = SRC_BF16 ? bf16_bits_to_f32(static_cast<const uint16_t *>(src)[i0 + e]) : static_cast<const float *>(src)[i0 + e];
  }
  uint32_t lo = 0, hi = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    if (e < m) {
      float t = rintf(__fmul_rn(v[e], scale));
      t = fminf(fmaxf(t, -127.f), 127.f);
      const uint32_t byte = (uint32_t)(int)t & 0xffu;
      if (e < 4) lo |= byte << (8 * e); else hi |= byte << (8 * (e - 4));
    }
  }
  if (m == 8) {
    *reinterpret_cast<uint2 *>(dst + i0) = make_uint2(lo, hi);
  } else {
    for (int e = 0; e < m; ++e) dst[i0 + e] = (int8_t)((e < 4 ? lo >> (8 * e) : hi >> (8 * (e - 4))) & 0xffu);
  }
}

extern "C" mol_status_t mol_quantize_int8(const void *src, int src_dtype, int64_t n, float scale, int8_t *dst,
                                          void *stream) {
  if (!src || !dst) return mol_fail(MOL_EINVAL, "mol_quantize_int8: src and dst must not be NULL");
  if (src_dtype != MOL_F32 && src_dtype != MOL_BF16) return mol_fail(MOL_EINVAL, "mol_quantize_int8: src_dtype must be MOL_F32 or MOL_BF16");
  if (n < 0 || !(scale > 0.f) || !isfinite(scale)) return mol_fail(MOL_EINVAL, "mol_quantize_int8: n >= 0 and a finite scale > 0 are required");
  if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 7u))
    return mol_fail(MOL_EINVAL, "mol_quantize_int8: src must be 16-byte and dst 8-byte aligned");
  if (n == 0) return MOL_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t threads = (n + 7) / 8;
  const unsigned grid = (unsigned)((threads + 255) / 256);
  if (src_dtype == MOL_BF16)
    hipLaunchKernelGGL(k_quantize_int8<true>, dim3(grid), dim3(256), 0, st, src, n, scale, dst);
  else
    hipLaunchKernelGGL(k_quantize_int8<false>, dim3(grid), dim3(256), 0, st, src, n, scale, dst);
  HIP_TRY(hipGetLastError());
  return MOL_OK;
}

extern "C" mol_status_t mol_corpus_free(mol_corpus_t *c) {
  if (!c) return MOL_OK;
  (void)hipDeviceSynchronize();
  if (c->w1c_frag_h && c->w1c_frag_h != c->w1c_frag) (void)hipFree(c->w1c_frag_h);
  if (c->w2_frag_h && c->w2_frag_h != c->w2_frag) (void)hipFree(c->w2_frag_h);
  if (c->w1c_frag) (void)hipFree(c->w1c_frag);
  if (c->w2_frag) (void)hipFree(c->w2_frag);
  if (c->w1u) (void)hipFree(c->w1u);
  if (c->b2) (void)hipFree(c->b2);
  if (c->xi) (void)hipFree(c->xi);
  if (c->xw) (void)hipFree(c->xw);
  if (c->wu1) (void)hipFree(c->wu1);
  if (c->wu2) (void)hipFree(c->wu2);
  if (c->bu1) (void)hipFree(c->bu1);
  if (c->bu2) (void)hipFree(c->bu2);
  if (c->b1c) (void)hipFree(c->b1c);
  if (c->seed) (void)hipFree(c->seed);
  if (c->wg1_frag) (void)hipFree(c->wg1_frag);
  if (c->wg2_frag) (void)hipFree(c->wg2_frag);
  if (c->bg1) (void)hipFree(c->bg1);
  if (c->bg2) (void)hipFree(c->bg2);
  if (c->own_stage1 && c->stage1) (void)hipFree(const_cast<void *>(c->stage1));
  if (c->own_embs && c->embs) (void)hipFree(const_cast<void *>(c->embs));
  free(c);
  return MOL_OK;
}
