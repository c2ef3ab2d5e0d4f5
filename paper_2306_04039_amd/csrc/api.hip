// C ABI entry points: argument checking, workspace carving, error reporting.
#include <stdarg.h>
#include <stdio.h>

#include "common.hpp"

static thread_local char g_err[512] = "";

mol_status_t mol_fail(mol_status_t st, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

extern "C" const char *mol_last_error(void) { return g_err; }

// ------------------------------------------------------------------------------------------------ timing
#include <mutex>
#include <vector>
namespace {
struct ProfRec {
  int slot;
  hipEvent_t a, b;
};
struct Prof {
  uint32_t mask = 0;  // bit s: slot s is timed
  std::mutex mu;
  std::vector<ProfRec> recs;
  std::vector<hipEvent_t> pool;
  hipEvent_t open_ev[MOL_PROF_SLOTS] = {};
  hipEvent_t get() {
    if (!pool.empty()) {
      hipEvent_t e = pool.back();
      pool.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
} g_prof;
}  // namespace

void mol_prof_begin(int slot, hipStream_t st) {
  if (!((g_prof.mask >> slot) & 1u)) return;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  hipEvent_t e = g_prof.get();
  if (e) (void)hipEventRecord(e, st);
  g_prof.open_ev[slot] = e;
}

void mol_prof_end(int slot, hipStream_t st) {
  if (!((g_prof.mask >> slot) & 1u)) return;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  hipEvent_t a = g_prof.open_ev[slot];
  g_prof.open_ev[slot] = nullptr;
  if (!a) return;
  hipEvent_t b = g_prof.get();
  if (!b) {
    g_prof.pool.push_back(a);
    return;
  }
  (void)hipEventRecord(b, st);
  g_prof.recs.push_back({slot, a, b});
}

extern "C" mol_status_t mol_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  g_prof.mask = on == 1 ? 0xffffffffu : (on <= 0 ? 0u : (uint32_t)on >> 1);
  return MOL_OK;
}

extern "C" mol_status_t mol_profile_read(double *slot_ms, int *slot_launches) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  double ms[MOL_PROF_SLOTS] = {};
  int n[MOL_PROF_SLOTS] = {};
  mol_status_t rc = MOL_OK;
  for (const ProfRec &r : g_prof.recs) {
    float t = 0.f;
    hipError_t e = hipEventSynchronize(r.b);
    if (e == hipSuccess) e = hipEventElapsedTime(&t, r.a, r.b);
    if (e != hipSuccess) rc = mol_fail(MOL_EHIP, "profile event: %s", hipGetErrorString(e));
    else {
      ms[r.slot] += t;
      n[r.slot] += 1;
    }
    g_prof.pool.push_back(r.a);
    g_prof.pool.push_back(r.b);
  }
  g_prof.recs.clear();
  for (int i = 0; i < MOL_PROF_SLOTS; ++i) {
    if (slot_ms) slot_ms[i] = ms[i];
    if (slot_launches) slot_launches[i] = n[i];
  }
  return rc;
}

extern "C" int64_t hindexer_default_lambda(const mol_corpus_t *c, int Kp) {
  if (!c || Kp < 1) return 0;
  const int64_t N = c->N;
  int64_t a = (N + 99) / 100;
  int64_t b = (256 * N + Kp - 1) / Kp;
  int64_t lam = a > b ? a : b;
  if (lam > N / 2) lam = N / 2;
  if (lam < 1) lam = 1;
  return lam;
}

extern "C" size_t hindexer_workspace_bytes(const mol_corpus_t *c, int B, int Kp, int64_t lambda) {
  if (!c || B < 1 || B > 1024 || Kp < 1 || Kp > c->N || c->d1 == 0) return 0;
  HindexerPlan p0, p1;
  if (hindexer_plan(c, B, Kp, lambda, MOL_HINDEXER_EXACT, &p0) != MOL_OK) return 0;
  if (hindexer_plan(c, B, Kp, lambda, MOL_HINDEXER_PAPER, &p1) != MOL_OK) return 0;
  return p0.total > p1.total ? p0.total : p1.total;
}

// U [B, H], UW [B, P], UP [B, H/32, 64] (the per-query inputs of the scoring kernels)
static size_t mol_user_bytes(const mol_corpus_t *c, int B) {
  return 3 * align_up((size_t)B * c->H * 4, 256) + align_up((size_t)B * c->P * 4, 256);
}
static void mol_user_ptrs(const mol_corpus_t *c, int B, char *ws, float **U, float **UW, uint32_t **UP) {
  *U = reinterpret_cast<float *>(ws);
  *UW = reinterpret_cast<float *>(ws + align_up((size_t)B * c->H * 4, 256));
  *UP = reinterpret_cast<uint32_t *>(ws + align_up((size_t)B * c->H * 4, 256) + align_up((size_t)B * c->P * 4, 256));
}

static size_t mol_ws_layout(const mol_corpus_t *c, int B, int64_t row, int k, size_t *off_scores, size_t *off_topk) {
  size_t off = mol_user_bytes(c, B);
  if (off_scores) *off_scores = off;
  off = align_up(off + (size_t)B * row * 4, 256);
  if (off_topk) *off_topk = off;
  off += final_topk_workspace_bytes(B, row, k);
  return off;
}

extern "C" size_t mol_workspace_bytes(const mol_corpus_t *c, int B, int Kp, int k) {
  if (!c || B < 1 || B > 1024 || k < 0) return 0;
  const int64_t row = Kp > 0 ? Kp : c->N;
  return mol_ws_layout(c, B, row, k, nullptr, nullptr);
}

static mol_status_t check_ws(const void *ws, size_t have, size_t need) {
  if (!ws) return mol_fail(MOL_EINVAL, "workspace is NULL (%zu bytes needed)", need);
  if (reinterpret_cast<uintptr_t>(ws) % 256) return mol_fail(MOL_EINVAL, "workspace must be 256-byte aligned");
  if (have < need) return mol_fail(MOL_EWORKSPACE, "workspace has %zu bytes, %zu needed", have, need);
  return MOL_OK;
}

// The kernels run on the current device: it has to be the one that holds the corpus.
static mol_status_t check_device(const mol_corpus_t *c) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev != c->device) return mol_fail(MOL_EINVAL, "the corpus lives on device %d but device %d is current", c->device, dev);
  return MOL_OK;
}

extern "C" mol_status_t hindexer_topk(const mol_corpus_t *c, const void *q1, int B, int Kp, const int32_t *sample_idx,
                                      int64_t lambda, uint64_t seed, int mode, int32_t *cand_idx, float *cand_score,
                                      int32_t *cand_count, void *workspace, size_t workspace_bytes, void *stream) {
  if (!c || !q1 || !cand_idx || !cand_count) return mol_fail(MOL_EINVAL, "hindexer_topk: NULL argument");
  if (c->d1 == 0 || !c->stage1) return mol_fail(MOL_EINVAL, "hindexer_topk: the corpus was packed without a stage-1 table");
  if (B < 1 || B > 1024) return mol_fail(MOL_EINVAL, "B=%d must be in [1, 1024]", B);
  if (Kp < 1 || Kp > c->N) return mol_fail(MOL_EINVAL, "Kp=%d must be in [1, N=%lld]", Kp, (long long)c->N);
  const int base_mode = mode & ~(MOL_HINDEXER_FORCE_REDO | MOL_HINDEXER_DEFER_REDO);
  if (base_mode != MOL_HINDEXER_EXACT && base_mode != MOL_HINDEXER_PAPER) return mol_fail(MOL_EINVAL, "unknown mode %d", mode);
  if (sample_idx && lambda < 1) return mol_fail(MOL_EINVAL, "an explicit sample needs lambda >= 1");
  HindexerPlan p;
  mol_status_t rc = check_device(c);
  if (rc != MOL_OK) return rc;
  rc = hindexer_plan(c, B, Kp, lambda, base_mode, &p);
  if (rc != MOL_OK) return rc;
  rc = check_ws(workspace, workspace_bytes, p.total);
  if (rc != MOL_OK) return rc;
  return hindexer_run(c, q1, B, Kp, sample_idx, seed, mode, p, cand_idx, cand_score, cand_count,
                      static_cast<char *>(workspace), static_cast<hipStream_t>(stream));
}

static mol_status_t mol_common_checks(const mol_corpus_t *c, const void *ue, const void *ug, int B,
                                      const int32_t *cand, int Kp) {
  if (!c || !ue || !ug) return mol_fail(MOL_EINVAL, "NULL corpus / user_embs / user_gate");
  if (B < 1 || B > 1024) return mol_fail(MOL_EINVAL, "B=%d must be in [1, 1024]", B);
  if (cand && Kp < 1) return mol_fail(MOL_EINVAL, "Kp=%d must be >= 1 when cand_idx is given", Kp);
  return check_device(c);
}

extern "C" mol_status_t mol_score(const mol_corpus_t *c, const void *user_embs, const void *user_gate, int B,
                                  const int32_t *cand_idx, int Kp, float *scores, void *workspace,
                                  size_t workspace_bytes, void *stream) {
  mol_status_t rc = mol_common_checks(c, user_embs, user_gate, B, cand_idx, Kp);
  if (rc != MOL_OK) return rc;
  if (!scores) return mol_fail(MOL_EINVAL, "scores is NULL");
  const size_t need = mol_user_bytes(c, B);
  rc = check_ws(workspace, workspace_bytes, need);
  if (rc != MOL_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  float *U, *UW;
  uint32_t *UP;
  mol_user_ptrs(c, B, static_cast<char *>(workspace), &U, &UW, &UP);
  if (cand_idx || !mol_exh_fast_form(c)) UP = nullptr;
  rc = launch_user_gate(c, user_gate, B, U, UW, UP, st);
  if (rc != MOL_OK) return rc;
  return launch_mol_score(c, user_embs, U, UW, UP, B, cand_idx, nullptr, Kp, scores, st);
}

extern "C" mol_status_t mol_gather_items(const mol_corpus_t *c, const int32_t *cand_idx, int B, int Kp, void *out_embs,
                                         void *stream) {
  if (!c || !cand_idx || !out_embs) return mol_fail(MOL_EINVAL, "mol_gather_items: NULL corpus / cand_idx / out_embs");
  if (B < 1 || B > 1024 || Kp < 1) return mol_fail(MOL_EINVAL, "mol_gather_items: B=%d must be in [1, 1024] and Kp=%d >= 1", B, Kp);
  if (reinterpret_cast<uintptr_t>(out_embs) & 15u) return mol_fail(MOL_EINVAL, "mol_gather_items: out_embs must be 16-byte aligned");
  const mol_status_t rc = check_device(c);
  if (rc != MOL_OK) return rc;
  return launch_gather_items(c, cand_idx, B, Kp, out_embs, static_cast<hipStream_t>(stream));
}

// Argument checks of mol_topk and the size of the workspace it needs.
static mol_status_t mol_topk_checks(const mol_corpus_t *c, const void *user_embs, const void *user_gate, int B,
                                    const int32_t *cand_idx, const int32_t *cand_count, int Kp, int k,
                                    const int32_t *out_idx, const float *out_score, size_t *need) {
  mol_status_t rc = mol_common_checks(c, user_embs, user_gate, B, cand_idx, Kp);
  if (rc != MOL_OK) return rc;
  if (!out_idx || !out_score) return mol_fail(MOL_EINVAL, "out_idx / out_score is NULL");
  if (k < 1 || k > 1024) return mol_fail(MOL_EINVAL, "k=%d must be in [1, 1024]", k);
  if (cand_count && !cand_idx) return mol_fail(MOL_EINVAL, "cand_count needs cand_idx");
  *need = mol_ws_layout(c, B, cand_idx ? Kp : c->N, k, nullptr, nullptr);
  return MOL_OK;
}

// The three launches of mol_topk on a workspace of mol_ws_layout's shape.
static mol_status_t mol_topk_run(const mol_corpus_t *c, const void *user_embs, const void *user_gate, int B,
                                 const int32_t *cand_idx, const int32_t *cand_count, int Kp, int k, int32_t *out_idx,
                                 float *out_score, char *ws, hipStream_t st) {
  const int64_t row = cand_idx ? Kp : c->N;
  size_t off_scores = 0, off_topk = 0;
  (void)mol_ws_layout(c, B, row, k, &off_scores, &off_topk);
  float *U, *UW;
  uint32_t *UP;
  mol_user_ptrs(c, B, ws, &U, &UW, &UP);
  if (cand_idx || !mol_exh_fast_form(c)) UP = nullptr;
  float *scores = reinterpret_cast<float *>(ws + off_scores);
  mol_status_t rc = launch_user_gate(c, user_gate, B, U, UW, UP, st);
  if (rc != MOL_OK) return rc;
  rc = launch_mol_score(c, user_embs, U, UW, UP, B, cand_idx, cand_count, row, scores, st);
  if (rc != MOL_OK) return rc;
  return launch_final_topk(scores, cand_idx, cand_count, B, row, k, out_idx, out_score, ws + off_topk, st);
}

extern "C" mol_status_t mol_topk(const mol_corpus_t *c, const void *user_embs, const void *user_gate, int B,
                                 const int32_t *cand_idx, const int32_t *cand_count, int Kp, int k, int32_t *out_idx,
                                 float *out_score, void *workspace, size_t workspace_bytes, void *stream) {
  size_t need = 0;
  mol_status_t rc = mol_topk_checks(c, user_embs, user_gate, B, cand_idx, cand_count, Kp, k, out_idx, out_score, &need);
  if (rc != MOL_OK) return rc;
  rc = check_ws(workspace, workspace_bytes, need);
  if (rc != MOL_OK) return rc;
  return mol_topk_run(c, user_embs, user_gate, B, cand_idx, cand_count, Kp, k, out_idx, out_score,
                      static_cast<char *>(workspace), static_cast<hipStream_t>(stream));
}

// ------------------------------------------------------------------------------------------------ no-allocation variant
// mol_topk for callers that cannot allocate (HIP graph capture, tight serving loops): the workspace of mol_topk -- U, UW,
// the [B, Kp] score matrix and the staging of the two-level selection -- lives in a file-scope device array.  Each GPU
// holds its own copy of the array at its own address; the address is looked up once per device and only that pointer is
// ever handed to kernels (the array's name is a host-side stand-in, not a device address).
static __device__ __align__(256) unsigned char scratch[MOL_TOPK_STATIC_MAX_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
unsigned char *g_scratch_ptr[kMaxDevices] = {};
}  // namespace

// Device address of `scratch` on the current device (resolved on the first call per device).
static mol_status_t scratch_for_current_device(unsigned char **out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return mol_fail(MOL_EUNSUPPORTED, "device ordinal %d is beyond %d", dev, kMaxDevices);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return mol_fail(MOL_EHIP, "hipGetSymbolAddress returned a null address for the static workspace");
    g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
  }
  *out = g_scratch_ptr[dev];
  return MOL_OK;
}

extern "C" mol_status_t mol_static_init(void) {
  unsigned char *p = nullptr;
  return scratch_for_current_device(&p);
}

extern "C" size_t mol_topk_static_max_bytes(void) { return MOL_TOPK_STATIC_MAX_BYTES; }

extern "C" mol_status_t mol_topk_static(const mol_corpus_t *c, const void *user_embs, const void *user_gate, int B,
                                        const int32_t *cand_idx, const int32_t *cand_count, int Kp, int k,
                                        int32_t *out_idx, float *out_score, void *stream) {
  size_t need = 0;
  mol_status_t rc = mol_topk_checks(c, user_embs, user_gate, B, cand_idx, cand_count, Kp, k, out_idx, out_score, &need);
  if (rc != MOL_OK) return rc;
  if (need > MOL_TOPK_STATIC_MAX_BYTES)
    return mol_fail(MOL_EWORKSPACE, "mol_topk_static: B=%d, row length %lld, k=%d need %zu bytes of workspace, the static one has %zu",
                    B, (long long)(cand_idx ? Kp : c->N), k, need, (size_t)MOL_TOPK_STATIC_MAX_BYTES);
  unsigned char *ws = nullptr;
  rc = scratch_for_current_device(&ws);
  if (rc != MOL_OK) return rc;
  // nothing in the workspace has to start at zero: U, UW, the scores and the staged candidates are all written in full by
  // the kernels before they are read, so what an earlier call left behind is never seen
  return mol_topk_run(c, user_embs, user_gate, B, cand_idx, cand_count, Kp, k, out_idx, out_score,
                      reinterpret_cast<char *>(ws), static_cast<hipStream_t>(stream));
}
