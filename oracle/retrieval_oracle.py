"""CPU oracle for two-stage retrieval: h-indexer (stage 1) + Mixture of Logits (stage 2).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module; it is
used by tests/, by the smoke check and by the benchmark's cpu_baseline leg.  It shares no
code, tables or helpers with the HIP library and is deliberately plain and slow:
fp64 arithmetic on the stored input bits (bf16 / fp32 widened exactly), sequential
definitions, full sorts, no blocking or fusion.

What it follows (paper sections, in the paper's notation):
  * stage-1 similarity and the filter loop: Algorithm 2 (h-indexer), Section 4.1.1 for the
    dot product itself.
  * the sampled threshold: Algorithm 2 (sample, nthElement at rank k/|data| * lambda, strict >),
    Section 4.1.2 for "up to k' items that meet the threshold".
  * component logits: Eq. 6 (all k_u x k_x pairwise dot products), Eq. 9 (division by tau, applied
    here as multiplication by logit_scale = 1/tau); the component index is user-major,
    p = ku * k_x + kx, the order Algorithm 1 hands the logits to the gate in.
  * gating: Eq. 8 / Section 3.2 (a network of item-side, user-side and cross inputs whose output is
    a probability distribution over the k_u*k_x components, Section 3.2 last paragraph), in the
    concrete form of the benchmark workloads: a 2-layer MLP on [component logits || user gate
    feature || item gate feature] followed by a softmax over the P components; and, as a second
    form, Algorithm 1's decomposedGating with the choices of Section 3.4 (three 2-layer MLPs,
    uw * xw + cw, SiLU, softmax).
  * similarity: Eq. 3 / Algorithm 1: phi = sum_p pi_p * cl_p, then the k best.

Readings where the paper is silent (ordering of equal scores, rank rounding, ...) are taken as:
total order (score descending, index ascending); threshold rank r_s = max(1, floor(k' * lambda / N)),
1-based from the largest; lambda is a count; the filter is strict.

Pins (tests/test_oracle_*.py): exact rational arithmetic for the dot product, brute-force top-k,
Algorithm 2 with the whole corpus as the sample, P = 1 reduces to the scaled dot product, gates sum
to one and phi lies between the smallest and largest component logit, a uniform gate gives the mean
logit in closed form, a user-only gate reproduces Eq. 5 through a different evaluation order, one-hot
gates expose the component index order, softmax shift invariance, a loop-by-loop re-derivation,
K' = N two-stage equals exhaustive MoL, corpus permutation and batch-split invariance; INT8 quantisation against
exact rational round-half-even on dyadic scales, hand-worked cases and hand-built values that separate "round the fp32
product" from "round the exact product" (the rule itself is the library's contract -- parity unpinned against the
paper, which gives no scheme), INT8 scores against Python integers;
Algorithm 1's decomposed gate: distribution / convexity, P = 1, all-zero heads give the mean logit, constant heads in
the two SiLU limits (softmax of the product; uniform), one-hot selection, scalar-loop re-derivation.
Generated item embeddings (Section 3.1): with a zero first layer every item gets the normalised bias, an identity MLP on
non-negative seeds returns the normalised seed chunks (both then equal the cached path on hand-built embeddings), unit
norm, invariance to a positive rescaling of the output layer, scalar-loop re-derivation.
The recall level of the approximate (sampled) mode is "parity unpinned": the paper's recall figure
carries no numbers.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

_MASK64 = (1 << 64) - 1


# --------------------------------------------------------------------------- input decoding
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Raw bfloat16 bit patterns (uint16) -> float64, exactly."""
    b = np.ascontiguousarray(bits)
    if b.dtype != np.uint16:
        raise TypeError("bf16 input must be given as uint16 bit patterns")
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def as_f64(a: np.ndarray) -> np.ndarray:
    """uint16 => bf16 bit patterns; float16/float32/float64 => widened; int8 => the integers (quantised stage-1 vectors)."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return bf16_bits_to_f64(a)
    if a.dtype in (np.float16, np.float32, np.float64, np.int8):
        return a.astype(np.float64)
    raise TypeError(f"unsupported input dtype {a.dtype}")


# --------------------------------------------------------------------------- ordering
def order_desc(scores: np.ndarray, ids: Optional[np.ndarray] = None) -> np.ndarray:
    """Permutation that sorts by (score descending, id ascending).  Full sort."""
    scores = np.asarray(scores, dtype=np.float64)
    ids = np.arange(scores.shape[0], dtype=np.int64) if ids is None else np.asarray(ids, dtype=np.int64)
    return np.lexsort((ids, -scores))


def topk_desc(scores: np.ndarray, k: int, ids: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """The k best entries under (score desc, id asc): returns (ids[k], scores[k])."""
    scores = np.asarray(scores, dtype=np.float64)
    ids = np.arange(scores.shape[0], dtype=np.int64) if ids is None else np.asarray(ids, dtype=np.int64)
    perm = order_desc(scores, ids)[: max(0, min(k, scores.shape[0]))]
    return ids[perm], scores[perm]


def nth_largest(values: np.ndarray, r: int) -> float:
    """r-th largest value, r counted from 1 (Algorithm 2, nthElement)."""
    v = np.sort(np.asarray(values, dtype=np.float64))[::-1]
    if not 1 <= r <= v.shape[0]:
        raise ValueError("rank out of range")
    return float(v[r - 1])


# --------------------------------------------------------------------------- stage 1
def quantize_int8(x: np.ndarray, scale: float) -> np.ndarray:
    """INT8 stage-1 vectors.  Section 4.1.1 names INT8 operands but no quantisation scheme, so this function is defined
    by the library's documented contract (its header), not by the paper: symmetric, one scale per tensor,
    q = clamp(round_half_even(fl32(x * scale)), -127, 127), where fl32 is ONE rounding of the product of the two fp32
    factors to fp32.  Rounding the product first matters only when the exact product lies within half an fp32 ulp of a
    half-integer; a pin separates the two rules on hand-built values.  PARITY UNPINNED against the paper for scales
    that are not powers of two: nothing in the paper fixes which of the two rules (or any other scheme) is meant."""
    xf = as_f64(x).astype(np.float32)                     # bf16 / fp32 inputs: exact
    t = (xf * np.float32(scale)).astype(np.float32)       # fp32 * fp32 -> fp32, rounded once
    return np.clip(np.rint(t), -127.0, 127.0).astype(np.int8)   # rint: halves to even


def stage1_scores(Q1: np.ndarray, X1: np.ndarray) -> np.ndarray:
    """s[b, n] = <Q1[b], X1[n]> in fp64 (Algorithm 2, dotProduct; Section 4.1.1).  For int8 inputs the result is the
    exact integer dot product (every product and every partial sum is an integer below 2^53), which is what the
    selection consumes: no scale is applied to it (Section 4.1.1)."""
    return as_f64(Q1) @ as_f64(X1).T


def exact_topk_stage1(Q1: np.ndarray, X1: np.ndarray, Kp: int) -> List[Tuple[np.ndarray, np.ndarray]]:
    """Exact top-K' per query: Algorithm 2 with the threshold replaced by the true K'-th score."""
    s = stage1_scores(Q1, X1)
    return [topk_desc(s[b], Kp) for b in range(s.shape[0])]


def splitmix64(x: int) -> int:
    """One step of the SplitMix64 output function applied to state x (x already advanced)."""
    z = x & _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def sample_indices(seed: int, lam: int, N: int) -> np.ndarray:
    """The library's documented sample: i-th index = floor(N * top32(SplitMix64 stream) / 2^32).

    The stream is the standard SplitMix64 sequence started at `seed` (state += 0x9E3779B97F4A7C15
    before each output).  Sampling is with replacement, which is harmless for a quantile estimate
    (Algorithm 2 uses the first lambda entries of a permutation).
    """
    i = np.arange(1, lam + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = np.uint64(seed & _MASK64) + i * np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return (((z >> np.uint64(32)) * np.uint64(N)) >> np.uint64(32)).astype(np.int64)


def threshold_rank(Kp: int, lam: int, N: int) -> int:
    """Rank of the sampled threshold: k/|data| * lambda, floored, at least 1 (Algorithm 2)."""
    return max(1, (Kp * lam) // N)


def hindexer(Q1: np.ndarray, X1: np.ndarray, Kp: int, sample_idx: Sequence[int], rank: Optional[int] = None,
             truncate: bool = True) -> List[Tuple[np.ndarray, np.ndarray, float]]:
    """Algorithm 2 for each query of a batch, with an explicit sample shared by the batch.

    Per query: scores of the sampled rows; t = the `rank`-th largest of them (default: the paper's
    rank); survivors = all n with s[n] > t (strict).  With `truncate`, more than K' survivors are cut
    to the K' best (Section 4.1.2: "up to k'").  Returns [(ids, scores, t)], ids ordered best first.
    """
    Xf, Qf = as_f64(X1), as_f64(Q1)
    N = Xf.shape[0]
    S = np.asarray(sample_idx, dtype=np.int64)
    r = threshold_rank(Kp, S.shape[0], N) if rank is None else rank
    out = []
    for b in range(Qf.shape[0]):
        s = Xf @ Qf[b]                      # dotProduct(x, query) for every x, computed once
        t = nth_largest(s[S], r)
        keep = np.nonzero(s > t)[0]
        ids, sc = topk_desc(s[keep], Kp if truncate else keep.shape[0], keep)
        out.append((ids, sc, t))
    return out


# --------------------------------------------------------------------------- stage 2 (MoL)
def _act(x: np.ndarray, act: str) -> np.ndarray:
    if act == "relu":
        return np.maximum(x, 0.0)
    if act == "silu":
        return x / (1.0 + np.exp(-x))
    raise ValueError(act)


def component_logits(F_b: np.ndarray, G_rows: np.ndarray, logit_scale: float) -> np.ndarray:
    """cl[c, p] = logit_scale * <F_b[ku], G_rows[c, kx]> for every pair (ku, kx)   (Eq. 6; Eq. 9 with 1/tau = logit_scale).

    F_b [k_u, d], G_rows [n, k_x, d] (fp64).  The component index is user-major, p = ku * k_x + kx: the order in which
    Algorithm 1 lays the k_u * k_x logits of one item out before they enter the gate.
    """
    k_u, _ = F_b.shape
    n, k_x, _ = G_rows.shape
    cl = np.empty((n, k_u * k_x), dtype=np.float64)
    for ku in range(k_u):
        for kx in range(k_x):
            cl[:, ku * k_x + kx] = logit_scale * (G_rows[:, kx, :] @ F_b[ku])
    return cl


def gating_weights(cl: np.ndarray, gu_b: np.ndarray, gx_rows: np.ndarray, W1: np.ndarray, b1: np.ndarray,
                   W2: np.ndarray, b2: np.ndarray, act: str = "relu") -> np.ndarray:
    """pi[c, :] = softmax(W2 * act(W1 * [cl[c] || gu_b || gx_rows[c]] + b1) + b2)   (Section 3.2)."""
    n = cl.shape[0]
    x = np.concatenate([cl, np.broadcast_to(gu_b, (n, gu_b.shape[0])), gx_rows], axis=1)
    h = _act(x @ W1.T + b1, act)
    z = h @ W2.T + b2
    z = z - z.max(axis=1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=1, keepdims=True)


def gather_items(G_bits: np.ndarray, cand: np.ndarray) -> np.ndarray:
    """Index select after the top-k' selection (Section 4.1.3): out[b, c] = the stored item row cand[b, c], bit for bit;
    a negative id (padding) gives an all-zero row.  G_bits [N, ...] of any dtype."""
    cand = np.asarray(cand, dtype=np.int64)
    out = np.zeros(cand.shape + G_bits.shape[1:], dtype=G_bits.dtype)
    for b in range(cand.shape[0]):
        for c in range(cand.shape[1]):
            if cand[b, c] >= 0:
                out[b, c] = G_bits[cand[b, c]]
    return out


def _mlp2(x: np.ndarray, Wa: np.ndarray, ba: np.ndarray, Wb: np.ndarray, bb: np.ndarray, act: str) -> np.ndarray:
    """Two-layer MLP, rows of x: Wb * act(Wa * x + ba) + bb."""
    return _act(x @ Wa.T + ba, act) @ Wb.T + bb


def decomposed_gating(cl: np.ndarray, gu_b: np.ndarray, gx_rows: np.ndarray, user_mlp, item_mlp, cross_mlp,
                      act: str = "relu") -> np.ndarray:
    """Algorithm 1, decomposedGating, with the choices Section 3.4 names: userWeightFn, itemWeightFn and crossWeightFn
    are 2-layer MLPs with k_u*k_x outputs; combineFn(uw, xw, cw) = uw * xw + cw (element-wise) followed by SiLU; then
    the softmax over the components.  Each *_mlp is (Wa, ba, Wb, bb); `act` is the MLPs' hidden nonlinearity (the paper
    does not name it)."""
    uw = _mlp2(gu_b[None, :], *user_mlp, act)          # uWeights      (1, P)
    xw = _mlp2(gx_rows, *item_mlp, act)                # xWeights      (n, P)   cachable
    cw = _mlp2(cl, *cross_mlp, act)                    # crossWeights  (n, P)
    z = _act(uw * xw + cw, "silu")                     # combineFn, then SiLU
    z = z - z.max(axis=1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=1, keepdims=True)


def generated_item_embeddings(seed_rows: np.ndarray, gen_mlp, k_g: int, d: int, act: str = "relu") -> np.ndarray:
    """Item-side embeddings produced at query time instead of being cached (Section 3.1, item-side bullet: some of the
    item-side embeddings are generated on the fly by learned MLPs, trading compute for accelerator memory).

    The paper fixes neither the MLP's input nor its depth; the reading taken: each item caches a small seed vector
    seed_rows[c] (d_s numbers); one 2-layer MLP (Wa [d_h, d_s], ba, Wb [k_g * d, d_h], bb) maps it to k_g vectors of
    length d, and each of them is L2-normalised like every other component embedding (Eq. 9; Algorithm 1's l2Norm):
        e = Wb * act(Wa * seed + ba) + bb,   g_j = e[j*d : (j+1)*d] / max(||e[j*d : (j+1)*d]||_2, 1e-12).
    Returns [n, k_g, d] (fp64)."""
    Wa, ba, Wb, bb = gen_mlp
    e = _mlp2(seed_rows, Wa, ba, Wb, bb, act).reshape(seed_rows.shape[0], k_g, d)
    norm = np.sqrt((e * e).sum(axis=2, keepdims=True))
    return e / np.maximum(norm, 1e-12)


class MolModelDecomposed:
    """Algorithm 1's gate (three 2-layer MLPs, multiplicative combination), decoded to fp64 once."""

    def __init__(self, G, gx, user_mlp, item_mlp, cross_mlp, logit_scale: float = 1.0, act: str = "relu"):
        self.G = as_f64(G)
        self.gx = as_f64(gx)
        dec = lambda m: tuple(as_f64(t) for t in m)
        self.user_mlp, self.item_mlp, self.cross_mlp = dec(user_mlp), dec(item_mlp), dec(cross_mlp)
        self.logit_scale = float(logit_scale)
        self.act = act


class MolModel:
    """Weights and item-side tensors, decoded to fp64 once."""

    def __init__(self, G, gx, W1, b1, W2, b2, logit_scale: float = 1.0, act: str = "relu", seed=None, gen_mlp=None):
        """seed [N, d_s] and gen_mlp (Wa, ba, Wb, bb): the last k_g = Wb.shape[0] / d item-side embeddings are generated
        from the seed (generated_item_embeddings) and follow the cached ones of G in the component order."""
        self.seed = None if seed is None else as_f64(seed)
        self.gen_mlp = None if gen_mlp is None else tuple(as_f64(t) for t in gen_mlp)
        self.G = as_f64(G)            # [N, k_x (cached), d]
        self.gx = as_f64(gx)          # [N, d_gx]
        self.W1 = as_f64(W1)          # [H, P + d_gu + d_gx]
        self.b1 = np.zeros(self.W1.shape[0]) if b1 is None else as_f64(b1)
        self.W2 = as_f64(W2)          # [P, H]
        self.b2 = np.zeros(self.W2.shape[0]) if b2 is None else as_f64(b2)
        self.logit_scale = float(logit_scale)
        self.act = act


def mol_scores_for(model: MolModel, F_b: np.ndarray, gu_b: np.ndarray, ids: np.ndarray,
                   chunk: int = 65536) -> np.ndarray:
    """phi(x, u) for one user and the listed items (Eq. 3 with Eq. 6 / Eq. 9 components)."""
    ids = np.asarray(ids, dtype=np.int64)
    out = np.empty(ids.shape[0], dtype=np.float64)
    for lo in range(0, ids.shape[0], chunk):
        sel = ids[lo: lo + chunk]
        G_rows = model.G[sel]
        if getattr(model, "gen_mlp", None) is not None:   # cached embeddings first, generated ones after them
            d = G_rows.shape[2]
            k_g = model.gen_mlp[2].shape[0] // d
            G_rows = np.concatenate([G_rows, generated_item_embeddings(model.seed[sel], model.gen_mlp, k_g, d, model.act)],
                                    axis=1)
        cl = component_logits(F_b, G_rows, model.logit_scale)
        if isinstance(model, MolModelDecomposed):
            pi = decomposed_gating(cl, gu_b, model.gx[sel], model.user_mlp, model.item_mlp, model.cross_mlp, model.act)
        else:
            pi = gating_weights(cl, gu_b, model.gx[sel], model.W1, model.b1, model.W2, model.b2, model.act)
        out[lo: lo + chunk] = (pi * cl).sum(axis=1)
    return out


def mol_scores(model: MolModel, F: np.ndarray, gu: np.ndarray, cand: Optional[np.ndarray] = None) -> np.ndarray:
    """Scores [B, K] for candidate ids cand[B, K] (negative id => -inf), or [B, N] when cand is None."""
    Ff, guf = as_f64(F), as_f64(gu)
    B = Ff.shape[0]
    N = model.G.shape[0]
    if cand is None:
        return np.stack([mol_scores_for(model, Ff[b], guf[b], np.arange(N)) for b in range(B)])
    cand = np.asarray(cand, dtype=np.int64)
    out = np.full(cand.shape, -np.inf, dtype=np.float64)
    for b in range(B):
        ok = cand[b] >= 0
        out[b, ok] = mol_scores_for(model, Ff[b], guf[b], cand[b, ok])
    return out


def mol_topk(model: MolModel, F: np.ndarray, gu: np.ndarray, cand: Optional[np.ndarray], k: int
             ) -> List[Tuple[np.ndarray, np.ndarray]]:
    """Algorithm 1's last step: the k most similar of the candidates (score desc, id asc)."""
    Ff, guf = as_f64(F), as_f64(gu)
    N = model.G.shape[0]
    out = []
    for b in range(Ff.shape[0]):
        ids = np.arange(N) if cand is None else np.asarray(cand[b], dtype=np.int64)
        ids = ids[ids >= 0]
        out.append(topk_desc(mol_scores_for(model, Ff[b], guf[b], ids), k, ids))
    return out


def two_stage(model: MolModel, Q1, X1, F, gu, Kp: int, k: int) -> List[Tuple[np.ndarray, np.ndarray]]:
    """Exact stage-1 top-K' followed by MoL top-k (the cascade of Section 2.2 with an exact first stage)."""
    stage1 = exact_topk_stage1(Q1, X1, Kp)
    cand = np.stack([ids for ids, _ in stage1])
    return mol_topk(model, F, gu, cand, k)
