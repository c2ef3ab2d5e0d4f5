// Memory-system ceilings, for benchmarks: what the device delivers to kernels that only move the bytes of the two
// bandwidth-bound steps and do no arithmetic on them.
//   * mol_bench_stream_read: a read-only sweep over a buffer (the stage-1 table of Section 4.1.1: every byte once), with
//                            streaming loads of whole lines, the fastest form found (7.1 TB/s; 6.3 with plain loads).
//   * mol_bench_gather     : the gather of the scoring kernel (Section 4.1.3) with its own lane-to-address mapping --
//                            per candidate the item's embedding block and its cached gate row -- and nothing else.
// Each thread folds what it loads into one word and stores it only if it equals a value that does not occur, so the
// loads cannot be dropped and nothing is written.
#include "common.hpp"

namespace {

__global__ __launch_bounds__(256) void k_stream_read(const uint4 *p, size_t n16, uint32_t *sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  uint32_t acc = 0;
  for (; i + 7 * stride < n16; i += 8 * stride) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = ld16_stream(p + i + u * stride);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n16; i += stride) {
    const uint4 v = ld16_stream(p + i);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9E3779B9u) sink[0] = acc;
}

// One wavefront per tile of 32 candidates of one query, as in the scoring kernel: lane (r16 = lane % 16, g = lane / 16)
// loads 16 bytes at offset 16 * g + 64 * s of row (candidate rt * CPR + r16 / K_X, component r16 % K_X); lane
// (c = lane % 32, h = lane / 32) loads 8-byte pieces of candidate c's cached gate row.  A wavefront keeps the loads of
// two tiles in flight (the scoring kernel overlaps the next tile's gathers with the current tile's arithmetic).
template <int K_X, int D_P, int H>
__global__ __launch_bounds__(256) void k_gather_bare(const char *embs, const char *xi, const int32_t *cand, int64_t Kp,
                                                     int B, int64_t N, uint32_t *sink) {
  constexpr int CPR = 16 / K_X, RT = 32 / CPR, SA = D_P / 32, XQ = H / 8;
  const int lane = threadIdx.x & 63;
  const int c = lane & 31, h = lane >> 5, r16 = lane & 15, g = lane >> 4;
  const int64_t tpq = (Kp + 31) >> 5;
  const int64_t ntiles = tpq * B;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  uint32_t acc = 0;
  auto tile_idx = [&](int64_t t) -> int {
    if (t >= ntiles) return 0;
    const int b = (int)(t / tpq);
    const int64_t pos = ((t % tpq) << 5) + c;
    const int idx = pos < Kp ? cand[(size_t)b * Kp + pos] : -1;
    return (idx < 0 || idx >= N) ? 0 : idx;
  };
  for (int64_t t = wave; t < ntiles; t += 2 * nwaves) {
    int idx[2] = {tile_idx(t), tile_idx(t + nwaves)};
    uint4 rows[2][RT][SA];
    uint2 gate[2][XQ];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        const int nidx = __shfl(idx[u], rt * CPR + r16 / K_X);
        const char *rowp = embs + (((size_t)nidx * K_X + (r16 % K_X)) * D_P + 8 * g) * 2;
#pragma unroll
        for (int s = 0; s < SA; ++s) rows[u][rt][s] = ld16(rowp + 64 * s);
      }
      if (xi) {
        const char *xp = xi + ((size_t)idx[u] * H + 4 * h) * 2;
#pragma unroll
        for (int o = 0; o < XQ; ++o) gate[u][o] = *reinterpret_cast<const uint2 *>(xp + 16 * o);
      } else {
#pragma unroll
        for (int o = 0; o < XQ; ++o) gate[u][o] = make_uint2(0u, 0u);
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int s = 0; s < SA; ++s) acc ^= rows[u][rt][s].x ^ rows[u][rt][s].y ^ rows[u][rt][s].z ^ rows[u][rt][s].w;
#pragma unroll
      for (int o = 0; o < XQ; ++o) acc ^= gate[u][o].x ^ gate[u][o].y;
    }
  }
  if (acc == 0x9E3779B9u) sink[0] = acc;
}

}  // namespace

extern "C" mol_status_t mol_bench_stream_read(const void *p, size_t bytes, int blocks, void *sink, void *stream) {
  if (!p || !sink || blocks < 1 || (reinterpret_cast<uintptr_t>(p) & 15u))
    return mol_fail(MOL_EINVAL, "mol_bench_stream_read: p (16-byte aligned), sink and blocks >= 1 are required");
  hipLaunchKernelGGL(k_stream_read, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4 *>(p), bytes / 16, static_cast<uint32_t *>(sink));
  HIP_TRY(hipGetLastError());
  return MOL_OK;
}

extern "C" mol_status_t mol_bench_gather(const mol_corpus_t *c, const int32_t *cand_idx, int B, int Kp, int blocks,
                                         void *sink, void *stream) {
  if (!c || !cand_idx || !sink || B < 1 || Kp < 1 || blocks < 1)
    return mol_fail(MOL_EINVAL, "mol_bench_gather: corpus, cand_idx, sink, B, Kp, blocks >= 1 are required");
  if (c->k_g > 0) return mol_fail(MOL_EUNSUPPORTED, "mol_bench_gather: not built for corpora with generated embeddings");
  const char *embs = static_cast<const char *>(c->embs), *xi = static_cast<const char *>(c->xi);
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint32_t *sk = static_cast<uint32_t *>(sink);
#define X(KU, KX, DP, HH)                                                                                           \
  if (c->k_x == KX && c->d_p == DP && c->H == HH) {                                                                 \
    hipLaunchKernelGGL((k_gather_bare<KX, DP, HH>), dim3((unsigned)blocks), dim3(256), 0, st, embs, xi, cand_idx,   \
                       (int64_t)Kp, B, c->N, sk);                                                                   \
    HIP_TRY(hipGetLastError());                                                                                     \
    return MOL_OK;                                                                                                  \
  }
  X(4, 4, 32, 32)
  X(4, 4, 64, 64)
  X(8, 4, 64, 128)
  X(8, 8, 64, 128)
  X(2, 8, 32, 64)
  X(16, 1, 32, 32)
  X(8, 2, 128, 96)
#undef X
  return mol_fail(MOL_EUNSUPPORTED, "mol_bench_gather: no instance for k_x=%d d_p=%d H=%d", c->k_x, c->d_p, c->H);
}
