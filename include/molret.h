/*
 * molret.h -- C ABI of the two-stage retrieval library for AMD MI355X (gfx950).
 *
 * The calls follow the paper's inference flow (Section 2.2, Figure 1(a)): an item-side cache is built
 * once (mol_corpus_pack); per query batch, stage 1 (h-indexer, Section 4.1, Algorithm 2) proposes K'
 * candidates per query from the whole corpus (hindexer_topk); stage 2 scores them with Mixture of
 * Logits (Section 3, Algorithm 1) (mol_score) and keeps the k best (mol_topk).
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer unless the comment says "host".  Tensors are row-major
 *     and contiguous.  bf16 tensors are raw 16-bit patterns ("bf16" below reads "fp16" for a corpus packed with
 *     mol_dtype = MOL_F16).  Item indices are int32 (N < 2^31).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work on it
 *     and return; none of them synchronises the device, except mol_corpus_pack / mol_corpus_free.
 *   - The caller owns all inputs, outputs and workspaces.  A corpus handle owns only what pack
 *     allocated.  Workspaces must be 256-byte aligned and at least as large as the matching
 *     *_workspace_bytes() call reports; their contents need not be preserved between calls.
 *   - Every function returns MOL_OK or a negative mol_status_t; mol_last_error() gives a message for
 *     the calling thread.  On MOL_EINVAL / MOL_EWORKSPACE / MOL_EUNSUPPORTED nothing was enqueued and
 *     outputs are untouched.  Nothing aborts or throws across this boundary.
 *   - Total order used everywhere: score descending, then item index ascending.
 */
#ifndef MOLRET_H
#define MOLRET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mol_corpus mol_corpus_t; /* opaque handle */

typedef enum {
  MOL_OK = 0,
  MOL_EINVAL = -1,       /* bad argument (null pointer, size out of range, misaligned workspace) */
  MOL_ENOMEM = -2,       /* device allocation failed in pack */
  MOL_EWORKSPACE = -3,   /* workspace too small */
  MOL_EUNSUPPORTED = -4, /* shape outside what the kernels are built for */
  MOL_EHIP = -5          /* a HIP runtime call failed */
} mol_status_t;

enum { MOL_F32 = 0, MOL_BF16 = 1, MOL_INT8 = 2, MOL_F16 = 3 }; /* stage1_dtype: F32, BF16 or INT8; mol_dtype: BF16 or F16 */
enum { MOL_ACT_RELU = 0, MOL_ACT_SILU = 1 }; /* act */
enum { MOL_GATE_CONCAT = 0, MOL_GATE_DECOMPOSED = 1 }; /* gate_form */

/* pack flags */
#define MOL_PACK_BORROW_STAGE1 1u /* keep the caller's stage-1 table (no copy); it must outlive the handle */
#define MOL_PACK_BORROW_EMBS 2u   /* keep the caller's item embedding tensor (no copy); same lifetime rule */

/* h-indexer modes */
#define MOL_HINDEXER_EXACT 0 /* sampled threshold at a deeper rank, exact top-K' of the survivors, exact redo on a miss */
#define MOL_HINDEXER_PAPER 1 /* Algorithm 2 as written: rank K'*lambda/N, strict filter, at most K' kept */
#define MOL_HINDEXER_FORCE_REDO 0x100 /* OR into mode: send every query through the exact radix redo (diagnostics, timing of an exact top-K');
                                         the result is that of the mode without the flag */
#define MOL_HINDEXER_DEFER_REDO 0x200 /* OR into mode: do not redo on the device.  A query the sample misled (or whose lists
                                         overflowed) comes back with cand_count[b] = -1 and an all -1 row, for the caller to
                                         submit again without this flag; every other query is unaffected.  Saves the nine
                                         launches of the redo, which return at once when no query needs them but still
                                         cost 15-40 us per call: for callers that read cand_count back anyway */

/*
 * Model description (host struct; read during mol_corpus_pack only).
 * Gating network (Section 3.2, Eq. 8, in the concatenated 2-layer form): for a (user, item) pair
 *   in  = [ cl (P = k_u*k_x component logits, index p = ku*k_x + kx) | user gate feature (d_gu) | item gate feature (d_gx) ]
 *   pi  = softmax_P( W2 * act(W1 * in + b1) + b2 ),    phi = sum_p pi_p * cl_p         (Eq. 3, Eq. 6)
 *   cl_p = logit_scale * <user_emb[ku], item_emb[kx]>                                   (Eq. 9; logit_scale = 1/tau)
 * Supported shapes: d1 = 64 (or 0); 1 <= d_gu <= 1024; d_gx in {16, 32, 64, 96, 128, 256}; (k_u, k_x, d_p, H) one of the combinations
 * the scoring kernel is instantiated for: (4,4,32,32), (4,4,64,64), (8,4,64,128), (8,8,64,128), (2,8,32,64),
 * (16,1,32,32), (8,2,128,96).  Anything else makes mol_corpus_pack return MOL_EUNSUPPORTED.
 */
typedef struct {
  int64_t N;            /* corpus size */
  int32_t d1;           /* stage-1 embedding width (Section 4.1.1); 0 = no stage-1 table */
  int32_t stage1_dtype; /* MOL_F32, MOL_BF16 or MOL_INT8 */
  int32_t k_u, k_x, d_p;
  int32_t d_gu, d_gx, H;
  int32_t act;
  float logit_scale;
  const void *W1;  /* device, bf16 [H, P + d_gu + d_gx] */
  const float *b1; /* device, f32 [H], or NULL for zeros */
  const void *W2;  /* device, bf16 [P, H] */
  const float *b2; /* device, f32 [P], or NULL for zeros */
  uint32_t flags;  /* MOL_PACK_* */
  /*
   * gate_form = MOL_GATE_DECOMPOSED selects Algorithm 1's decomposedGating with the choices of Section 3.4 instead of
   * the concatenated MLP above:
   *   uw = Wu2 * act(Wu1 * user_gate + bu1) + bu2      (userWeightFn, once per query)
   *   xw = Wx2 * act(Wx1 * item_gate + bx1) + bx2      (itemWeightFn, cached per item by mol_corpus_pack as f32 [N, P])
   *   cw = W2  * act(W1  * cl        + b1 ) + b2       (crossWeightFn; W1 is then bf16 [H, P])
   *   pi = softmax_P( SiLU( uw * xw + cw ) ),   phi = sum_p pi_p * cl_p
   * All second layers have P outputs; 16 <= d_hu, d_hx <= 1024.  Zero-initialise the struct to get MOL_GATE_CONCAT.
   */
  int32_t gate_form;
  int32_t d_hu, d_hx; /* hidden widths of the user and item weight MLPs */
  const void *Wu1;  /* device, bf16 [d_hu, d_gu] */
  const float *bu1; /* device, f32 [d_hu] or NULL */
  const void *Wu2;  /* device, bf16 [P, d_hu] */
  const float *bu2; /* device, f32 [P] or NULL */
  const void *Wx1;  /* device, bf16 [d_hx, d_gx] */
  const float *bx1; /* device, f32 [d_hx] or NULL */
  const void *Wx2;  /* device, bf16 [P, d_hx] */
  const float *bx2; /* device, f32 [P] or NULL */
  /*
   * mol_dtype = MOL_F16: every 16-bit tensor of stage 2 (item_embs, item_gate, all weight matrices here, and user_embs /
   * user_gate in mol_score / mol_topk, the output of mol_gather_items) is IEEE half instead of bfloat16 -- Section 4.3
   * serves in FP16; a model trained in BF16 converts to it without rounding.  0 or MOL_BF16 = bfloat16.
   */
  int32_t mol_dtype;
  /*
   * Item-side embeddings generated on the fly (Section 3.1, item-side bullet: accelerator memory limits how many item
   * embeddings can be cached, so some are produced at query time by a learned MLP, trading compute for memory).
   * k_x_gen > 0: of the k_x item-side embeddings of an item only the first k_x - k_x_gen are cached (item_embs is then
   * bf16 [N, k_x - k_x_gen, d_p]); the last k_x_gen are computed inside the scoring kernel for every candidate:
   *   e   = Wg2 * act(Wg1 * item_seed[n] + bg1) + bg2            (k_x_gen * d_p numbers)
   *   g_j = e[j*d_p : (j+1)*d_p] / max(||.||_2, 1e-12)            (Eq. 9: every component embedding is L2-normalised)
   * and take the places k_x - k_x_gen .. k_x - 1 in the item-side component order.  The seed, both weight matrices and the
   * hidden units enter the matrix cores as IEEE half (bf16 inputs convert exactly), the generated embeddings are rounded
   * once to half.  Concatenated gate only; (k_u, k_x, d_p, H, k_x_gen, d_s, d_hg) must be one of
   * (4,4,64,64,2,32,64), (8,8,64,128,2,32,64), else MOL_EUNSUPPORTED.  mol_gather_items returns the cached embeddings.
   */
  int32_t k_x_gen;       /* 0 = every item-side embedding is cached */
  int32_t d_s, d_hg;     /* seed width, hidden width of the generator */
  const void *item_seed; /* device, bf16 [N, d_s]; copied (as half) by mol_corpus_pack */
  const void *Wg1;       /* device, bf16 [d_hg, d_s] */
  const float *bg1;      /* device, f32 [d_hg] or NULL */
  const void *Wg2;       /* device, bf16 [k_x_gen * d_p, d_hg] */
  const float *bg2;      /* device, f32 [k_x_gen * d_p] or NULL */
} mol_config_t;

/*
 * Build the item-side cache (Section 2.2: whatever depends on the item alone is computed once and kept; the loops
 * marked cachable in Algorithm 1): keeps the stage-1 table [N, d1] and the item component embeddings [N, k_x, d_p] (already
 * L2-normalised by the caller, Eq. 9), and precomputes the item half of the first gating layer,
 * Xi[n] = W1[:, P+d_gu:] * item_gate[n] + b1, stored as bf16 [N, H] (decomposed gate: the item weights xw, f32 [N, P]).
 *   stage1_items : [N, d1] of stage1_dtype (fp32, bf16 or int8), or NULL when cfg->d1 == 0 (MoL-only use, Section 5.2.1 K' = X).
 *   item_embs    : bf16 [N, k_x, d_p] ([N, k_x - k_x_gen, d_p] with generated embeddings).
 *   item_gate    : bf16 [N, d_gx]; not referenced after the call returns.
 * Allocates device memory with hipMalloc; synchronises `stream` before returning.  *out is set on MOL_OK only.
 */
mol_status_t mol_corpus_pack(const mol_config_t *cfg, const void *stage1_items, const void *item_embs,
                             const void *item_gate, void *stream, mol_corpus_t **out);

/*
 * INT8 stage 1 (Section 4.1.1: the stage-1 dot product runs on INT8 operands and its INT32 result goes to the selection
 * without a de-quantising scale).  A corpus packed with stage1_dtype = MOL_INT8 takes stage1_items as int8 [N, 64] and
 * hindexer_topk then takes q1 as int8 [B, 64]; scores are exact integers (|s| <= 64*127*127), reported in cand_score as
 * floats holding those integers.  This helper produces such tensors with one symmetric scale per call:
 *   dst[i] = clamp(rint(src[i] * scale), -127, 127), the product rounded once to fp32, halves rounded to even.
 *   src : n elements of src_dtype (MOL_F32 or MOL_BF16), 16-byte aligned.   dst : int8 [n], 8-byte aligned.
 * A common choice is scale = 127 / max|src|; any positive scale keeps the order of one query's scores up to rounding.
 */
mol_status_t mol_quantize_int8(const void *src, int src_dtype, int64_t n, float scale, int8_t *dst, void *stream);

/* Frees what pack allocated (device synchronising).  NULL is accepted. */
mol_status_t mol_corpus_free(mol_corpus_t *corpus);

/* Size queries (no device work); return 0 on invalid arguments.  lambda <= 0 selects the default sample size.  The first
 * hindexer_workspace_bytes / hindexer_topk call of a process asks the HIP runtime for the occupancy of the scan kernels
 * (once per kernel variant; later calls make no runtime queries), so the device the corpus lives on must be current. */
size_t hindexer_workspace_bytes(const mol_corpus_t *corpus, int B, int Kp, int64_t lambda);
size_t mol_workspace_bytes(const mol_corpus_t *corpus, int B, int Kp, int k);

/* Default sample size for (N, K'): max(ceil(0.01 N), ceil(256 N / K')), capped at N/2 (Section 4.1.2: r in [0.01, 0.1]). */
int64_t hindexer_default_lambda(const mol_corpus_t *corpus, int Kp);

/*
 * Stage 1 (Algorithm 2; Sections 4.1.1-4.1.2): for each of B queries, score `lambda` sampled items, take the
 * sampled score of rank r as threshold t_b, stream the whole stage-1 table once computing <q1[b], x[n]> for all
 * b and n, keep (n, score) with score > t_b (strict), and reduce the survivors to at most K' candidates.
 *   q1          : [B, d1] of the corpus' stage1_dtype.   1 <= B <= 1024, 1 <= Kp <= N.
 *   sample_idx  : int32 [lambda] explicit sample (each in [0, N)), or NULL: the library then draws
 *                 idx_i = floor(N * hi32(SplitMix64_i(seed)) / 2^32), i = 1..lambda (stream state seed + i*0x9E3779B97F4A7C15).
 *   lambda      : sample size (a count); <= 0 = hindexer_default_lambda(); values above N are taken as N (of an
 *                 explicit sample the first N entries are used).  Ignored when 4*Kp >= N (no sampling: every
 *                 item passes and the exact top-K' is taken).
 *   mode        : MOL_HINDEXER_PAPER  r = max(1, floor(Kp*lambda/N)); more than K' survivors are cut to the K' best,
 *                                     fewer are returned as they are (cand_count[b] < Kp).  A query whose survivors
 *                                     overflow the workspace lists (items above the threshold packed into a few
 *                                     neighbouring rows) is redone on the device and gives the same set: the K' best
 *                                     that lie above t_b.
 *                 MOL_HINDEXER_EXACT  r = r_paper + ceil(5*sqrt(r_paper)) + 8 so that at least K' survive (the threshold is
 *                                     the rank-r sampled score or a value just below it: only the result is defined in
 *                                     this mode, and a lower threshold cannot change it), then the exact
 *                                     top-K' of the survivors; a query whose survivors number fewer than K' or overflow the
 *                                     workspace is redone on the device with an exact multi-pass radix threshold.  The
 *                                     result is the exact stage-1 top-K' under fp32 scores.  cand_count[b] = -1 (row
 *                                     all -1) reports a query that could not be completed; it does not occur for
 *                                     finite scores.
 *                 | MOL_HINDEXER_DEFER_REDO (either mode): the device redo is not run; a query that needs it is reported
 *                                     with cand_count[b] = -1 and is to be submitted again without the flag.
 *                 | MOL_HINDEXER_FORCE_REDO (either mode): every query takes the redo (same result; diagnostics).
 *   cand_idx    : out int32 [B, Kp]; a set, in no particular order; unused slots are -1.
 *   cand_score  : out f32 [B, Kp] stage-1 scores aligned with cand_idx (unused slots -inf), or NULL.
 *   cand_count  : out int32 [B] number of valid slots.
 * Scores are fp32 accumulations of the stored bf16 / fp32 values; exact integers for an int8 table.
 */
mol_status_t hindexer_topk(const mol_corpus_t *corpus, const void *q1, int B, int Kp, const int32_t *sample_idx,
                           int64_t lambda, uint64_t seed, int mode, int32_t *cand_idx, float *cand_score,
                           int32_t *cand_count, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Stage 2 scores (Algorithm 1 without its last line; Eq. 3, 6, 9; gating as described at mol_config_t).
 *   user_embs : bf16 [B, k_u, d_p] (L2-normalised by the caller).   user_gate : bf16 [B, d_gu].
 *   cand_idx  : int32 [B, Kp] item indices, negative = padding (score -inf); or NULL = every item 0..N-1 for
 *               every query (Kp is then ignored and the row length is N).
 *   scores    : out f32 [B, Kp] (or [B, N]).
 * Component logits, both gating layers, the softmax and the weighted sum run in one kernel; logits and hidden
 * activations enter the matrix cores as bf16, accumulation and the final sum are fp32.
 */
mol_status_t mol_score(const mol_corpus_t *corpus, const void *user_embs, const void *user_gate, int B,
                       const int32_t *cand_idx, int Kp, float *scores, void *workspace, size_t workspace_bytes,
                       void *stream);

/*
 * Index select (Section 4.1.3), for callers that want the candidates' embeddings themselves (mol_score / mol_topk gather
 * inside the scoring kernel and never materialise this tensor).
 *   cand_idx : int32 [B, Kp], negative = padding.
 *   out_embs : out bf16 [B, Kp, k_x, d_p], 16-byte aligned: a bit-exact copy of item row cand_idx[b, c]; zeros for padding.
 */
mol_status_t mol_gather_items(const mol_corpus_t *corpus, const int32_t *cand_idx, int B, int Kp, void *out_embs,
                              void *stream);

/*
 * Stage 2 with the final selection (Algorithm 1 including its last line): the k best candidates per query.
 *   cand_idx / Kp as in mol_score (NULL = exhaustive MoL over the corpus).
 *   cand_count: int32 [B] or NULL.  When given (hindexer_topk's output of that name), only the first cand_count[b] slots
 *               of row b are read -- the rest of the row is neither scored nor gathered, whatever it holds; a negative
 *               count reads as 0.  NULL = all Kp slots (negative entries are still padding).  Needs cand_idx.
 *   out_idx   : out int32 [B, k] item indices, best first (score desc, index asc); -1 where fewer than k exist.  An
 *               item that a row names more than once is a candidate as often as it is named (and can be returned so).
 *   out_score : out f32 [B, k] their MoL scores (-inf padding).
 */
mol_status_t mol_topk(const mol_corpus_t *corpus, const void *user_embs, const void *user_gate, int B,
                      const int32_t *cand_idx, const int32_t *cand_count, int Kp, int k, int32_t *out_idx,
                      float *out_score, void *workspace, size_t workspace_bytes, void *stream);

/*
 * mol_topk for callers that cannot allocate device memory or supply a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, results and kernels as mol_topk, minus the workspace:
 * the per-query gate inputs, the [B, Kp] score matrix and the staging of the final selection live in a static device
 * array of MOL_TOPK_STATIC_MAX_BYTES that every GPU the library runs on holds until the process ends.
 *   - Calls nothing that allocates (no hipMalloc / hipFree, no library allocation); enqueues on `stream` and returns.
 *   - MOL_EWORKSPACE when mol_workspace_bytes(corpus, B, Kp, k) exceeds MOL_TOPK_STATIC_MAX_BYTES (the 100M-item
 *     workload, B = 32, Kp = 100000, k = 100, needs 13.1 MB); nothing is enqueued then.
 *   - All calls on one GPU share that GPU's array: two calls whose kernels may overlap (different streams, or one stream
 *     captured into graphs replayed concurrently) race; callers serialise them.  The contents left by one call are never
 *     read by the next (every buffer is written in full before it is read), so nothing needs clearing between calls.
 *   - The array's device address is looked up on the first call on each device (hipGetSymbolAddress, which may load
 *     the code object); mol_static_init() does the lookup for the current device ahead of time, e.g. before a capture.
 */
#define MOL_TOPK_STATIC_MAX_BYTES (16u << 20)
mol_status_t mol_static_init(void);
size_t mol_topk_static_max_bytes(void);
mol_status_t mol_topk_static(const mol_corpus_t *corpus, const void *user_embs, const void *user_gate, int B,
                             const int32_t *cand_idx, const int32_t *cand_count, int Kp, int k, int32_t *out_idx,
                             float *out_score, void *stream);

/*
 * Optional per-kernel timing, for benchmarks.  While enabled, the kernel launches of the calls above are bracketed by
 * HIP events on the caller's stream (each bracket costs about 10 microseconds of idle device time).  mol_profile_read
 * synchronises on the recorded events, adds up the elapsed time per slot since the last read and clears the record.
 *   on : 0 = off, 1 = every slot, otherwise 2 * m where bit s of m enables slot s (e.g. 2 << MOL_PROF_SCAN_FILTER
 *        times the corpus scan only).
 *   slot_ms, slot_launches : host arrays of MOL_PROF_SLOTS entries (either may be NULL).
 */
enum {
  MOL_PROF_SAMPLE_SCORES = 0, /* stage 1: scores of the sampled rows */
  MOL_PROF_THRESHOLD = 1,     /* stage 1: per-query sampled threshold */
  MOL_PROF_SCAN_FILTER = 2,   /* stage 1: corpus scan + threshold filter */
  MOL_PROF_SELECT = 3,        /* stage 1: survivors -> K' candidates (and the exact redo, when taken) */
  MOL_PROF_USER_GATE = 4,     /* stage 2: user half of gating layer 1 */
  MOL_PROF_MOL_SCORE = 5,     /* stage 2: fused gather + component logits + gating + softmax + sum */
  MOL_PROF_FINAL_TOPK = 6,    /* stage 2: k best */
  MOL_PROF_SLOTS = 8
};
mol_status_t mol_profile_enable(int on);
mol_status_t mol_profile_read(double *slot_ms, int *slot_launches);

/*
 * Memory-system ceilings, for benchmarks (no arithmetic; nothing is written): the time these take is what the device
 * delivers to any kernel that has to move the same bytes.
 *   mol_bench_stream_read : reads `bytes` (a multiple of 16) from p once, front to back, with `blocks` workgroups of 256
 *                           threads -- the traffic of the stage-1 corpus scan (Section 4.1.1).
 *   mol_bench_gather      : for every candidate of cand_idx [B, Kp] reads the item's embedding block and cached gate row
 *                           with the lane-to-address mapping of the scoring kernel (Section 4.1.3) -- the traffic of
 *                           mol_score.  Negative / out-of-range ids read item 0.
 *   sink : device, 4 bytes, never written in practice (it keeps the loads alive).
 */
mol_status_t mol_bench_stream_read(const void *p, size_t bytes, int blocks, void *sink, void *stream);
mol_status_t mol_bench_gather(const mol_corpus_t *corpus, const int32_t *cand_idx, int B, int Kp, int blocks, void *sink,
                              void *stream);

/* Message for the last non-OK status returned on this thread (host string, valid until the next call). */
const char *mol_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MOLRET_H */
