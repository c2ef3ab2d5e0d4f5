"""Pins for the CPU oracle: each check ties one oracle function to something other than itself
(exact rational arithmetic, brute force, closed forms and special cases stated in the paper)."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import retrieval_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers
def rand_bf16_bits(rng, shape, scale=1.0):
    """Random bf16 bit patterns (uint16): fp32 normals truncated to their upper 16 bits."""
    x = (rng.standard_normal(shape) * scale).astype(np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16)


def bf16_fraction(bits: int) -> Fraction:
    """Decode one bf16 bit pattern by hand (sign, 8-bit exponent, 7-bit mantissa) to an exact rational."""
    sign = -1 if bits >> 15 else 1
    e = (bits >> 7) & 0xFF
    m = bits & 0x7F
    assert e != 0xFF
    if e == 0:
        return sign * Fraction(m, 1 << 7) * Fraction(1, 1 << 126)
    return sign * (1 + Fraction(m, 1 << 7)) * (Fraction(2) ** (e - 127))


def unit_rows(x):
    return x / np.linalg.norm(x, axis=-1, keepdims=True)


def small_model(rng, N=40, k_u=2, k_x=3, d=8, H=5, d_gu=4, d_gx=3, scale=1.0, act="relu", bias=True):
    P = k_u * k_x
    G = rand_bf16_bits(rng, (N, k_x, d), 0.5)
    gx = rand_bf16_bits(rng, (N, d_gx), 0.5)
    W1 = rand_bf16_bits(rng, (H, P + d_gu + d_gx), 0.7)
    W2 = rand_bf16_bits(rng, (P, H), 0.7)
    b1 = (rng.standard_normal(H) * 0.3).astype(np.float32) if bias else None
    b2 = (rng.standard_normal(P) * 0.3).astype(np.float32) if bias else None
    model = orc.MolModel(G, gx, W1, b1, W2, b2, logit_scale=scale, act=act)
    F = rand_bf16_bits(rng, (3, k_u, d), 0.5)
    gu = rand_bf16_bits(rng, (3, d_gu), 0.5)
    return model, F, gu


# ----------------------------------------------------------------------------- decoding + dot product
def test_bf16_decode_matches_hand_decoding():
    rng = np.random.default_rng(0)
    bits = rand_bf16_bits(rng, (200,), 3.0)
    bits[:4] = [0x0000, 0x8000, 0x3F80, 0x0001]          # +0, -0, 1.0, smallest subnormal
    got = orc.bf16_bits_to_f64(bits)
    for b, g in zip(bits.tolist(), got.tolist()):
        assert Fraction(g) == bf16_fraction(b)


def test_stage1_scores_exact_rational():
    """Products of bf16 values and their 16-term sums are exactly representable in fp64 here,
    so the oracle's dot product must equal exact rational arithmetic."""
    rng = np.random.default_rng(1)
    Q = rand_bf16_bits(rng, (3, 16))
    X = rand_bf16_bits(rng, (7, 16))
    s = orc.stage1_scores(Q, X)
    assert s.shape == (3, 7)
    for b in range(3):
        for n in range(7):
            exact = sum(bf16_fraction(int(Q[b, j])) * bf16_fraction(int(X[n, j])) for j in range(16))
            assert abs(Fraction(s[b, n]) - exact) <= abs(exact) * Fraction(1, 10**14)


def test_stage1_scores_orientation_fp32():
    Q = np.array([[1, 0, 0], [0, 2, 0]], dtype=np.float32)
    X = np.array([[3, 5, 7], [11, 13, 17], [19, 23, 29], [1, 1, 1]], dtype=np.float32)
    s = orc.stage1_scores(Q, X)
    assert s.tolist() == [[3, 11, 19, 1], [10, 26, 46, 2]]


# ----------------------------------------------------------------------------- ordering / top-k
def brute_topk(scores, ids, k):
    """Repeated arg-max with removal; ties broken by the smaller id."""
    pool = list(zip(scores, ids))
    out = []
    for _ in range(min(k, len(pool))):
        best = 0
        for i in range(1, len(pool)):
            if pool[i][0] > pool[best][0] or (pool[i][0] == pool[best][0] and pool[i][1] < pool[best][1]):
                best = i
        out.append(pool.pop(best))
    return [i for _, i in out], [s for s, _ in out]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_topk_matches_brute_force_with_ties(seed):
    rng = np.random.default_rng(seed)
    scores = rng.integers(0, 12, size=300).astype(np.float64) / 4.0       # many exact ties
    ids = rng.permutation(1000)[:300]
    for k in (1, 7, 100, 300, 400):
        gi, gs = orc.topk_desc(scores, k, ids)
        bi, bs = brute_topk(scores.tolist(), ids.tolist(), k)
        assert gi.tolist() == bi and gs.tolist() == bs


def test_nth_largest_is_one_based_from_the_top():
    v = np.array([5.0, 1.0, 9.0, 7.0, 7.0])
    assert orc.nth_largest(v, 1) == 9.0
    assert orc.nth_largest(v, 2) == 7.0
    assert orc.nth_largest(v, 3) == 7.0
    assert orc.nth_largest(v, 5) == 1.0
    with pytest.raises(ValueError):
        orc.nth_largest(v, 0)


# ----------------------------------------------------------------------------- sampler
def test_splitmix64_published_vector():
    want = [int(line) for line in open(os.path.join(GOLDEN, "splitmix64_seed1234567.txt")) if line[0].isdigit()]
    state, got = 1234567, []
    for _ in want:
        state = (state + 0x9E3779B97F4A7C15) & ((1 << 64) - 1)
        got.append(orc.splitmix64(state))
    assert got == want


def test_sample_indices_vectorised_equals_scalar_and_is_uniform():
    N, lam, seed = 1000, 20000, 77
    got = orc.sample_indices(seed, lam, N)
    state = seed
    for i in range(50):
        state = (state + 0x9E3779B97F4A7C15) & ((1 << 64) - 1)
        assert got[i] == ((orc.splitmix64(state) >> 32) * N) >> 32
    assert got.min() >= 0 and got.max() < N
    counts = np.bincount(got, minlength=N)
    # mean 20 per bin, std ~4.5: a broken mapping (e.g. only low indices) fails this by far
    assert counts.min() > 0 and counts.max() < 60
    assert abs(got.mean() - (N - 1) / 2) < 10


def test_threshold_rank():
    assert orc.threshold_rank(100_000, 1_000_000, 100_000_000) == 1000
    assert orc.threshold_rank(10, 10, 1000) == 1            # never below 1
    assert orc.threshold_rank(1024, 25_000, 100_000) == 256


# ----------------------------------------------------------------------------- Algorithm 2
def test_hindexer_full_sample_is_exact_threshold():
    """Sample = whole corpus and rank = K': t is the K'-th largest score, so the strict filter keeps
    exactly the items strictly above it (K'-1 of them when scores are distinct)."""
    rng = np.random.default_rng(3)
    Q = rng.integers(-8, 9, size=(2, 8)).astype(np.float32)          # integer data: every dot product exact
    X = rng.integers(-8, 9, size=(500, 8)).astype(np.float32)
    Kp = 37
    res = orc.hindexer(Q, X, Kp, np.arange(500))
    for b, (ids, sc, t) in enumerate(res):
        s = [sum(int(Q[b, j]) * int(X[n, j]) for j in range(8)) for n in range(500)]
        order = sorted(range(500), key=lambda n: (-s[n], n))
        assert t == s[order[Kp - 1]]
        above = [n for n in order if s[n] > t]                        # strict: ties with t are dropped
        assert len(above) <= Kp - 1
        assert ids.tolist() == above
        assert np.all(sc > t)


def test_hindexer_general_sample_invariants_and_truncation():
    rng = np.random.default_rng(4)
    Q = rng.integers(-8, 9, size=(3, 8)).astype(np.float32)
    X = rng.integers(-8, 9, size=(2000, 8)).astype(np.float32)
    S = orc.sample_indices(5, 400, 2000)
    Kp = 100                                              # rank = 100*400/2000 = 20
    full = orc.hindexer(Q, X, Kp, S, truncate=False)
    cut = orc.hindexer(Q, X, Kp, S, truncate=True)
    s = np.array([[sum(int(Q[b, j]) * int(X[n, j]) for j in range(8)) for n in range(2000)] for b in range(3)],
                 dtype=np.float64)
    for b in range(3):
        ids, sc, t = full[b]
        assert t == np.sort(s[b, S])[::-1][19]
        assert set(ids.tolist()) == {n for n in range(2000) if s[b, n] > t}
        cids, csc, _ = cut[b]
        assert len(cids) == min(Kp, len(ids)) and cids.tolist() == ids[: len(cids)].tolist()
        assert np.all(np.diff(csc) <= 0)
        # the estimate is in the right region: expected count K', binomial spread ~ K'/sqrt(rank)
        assert 30 <= len(ids) <= 250


def test_hindexer_deeper_rank_keeps_superset():
    rng = np.random.default_rng(5)
    Q = rng.standard_normal((1, 8)).astype(np.float32)
    X = rng.standard_normal((1000, 8)).astype(np.float32)
    S = orc.sample_indices(9, 300, 1000)
    a = orc.hindexer(Q, X, 50, S, rank=10, truncate=False)[0][0]
    b = orc.hindexer(Q, X, 50, S, rank=25, truncate=False)[0][0]
    assert set(a.tolist()) <= set(b.tolist())


# ----------------------------------------------------------------------------- MoL
def test_component_index_is_user_major():
    """Algorithm 1's view/permute: component p = ku * k_x + kx."""
    rng = np.random.default_rng(6)
    F = rng.standard_normal((3, 5))
    G = rng.standard_normal((4, 2, 5))
    cl = orc.component_logits(F, G, 0.5)
    assert cl.shape == (4, 6)
    for c in range(4):
        for ku in range(3):
            for kx in range(2):
                want = 0.5 * sum(F[ku, j] * G[c, kx, j] for j in range(5))
                assert abs(cl[c, ku * 2 + kx] - want) < 1e-14


def test_mol_single_component_is_scaled_dot_product():
    """P = 1: the softmax over one component is 1, so phi = <f, g> / tau (Eq. 4 with one term, Eq. 9)."""
    rng = np.random.default_rng(7)
    model, F, gu = small_model(rng, k_u=1, k_x=1, scale=1 / 20)
    phi = orc.mol_scores(model, F, gu)
    Ff, Gf = orc.as_f64(F), model.G
    want = np.einsum("bd,nd->bn", Ff[:, 0], Gf[:, 0]) / 20
    np.testing.assert_allclose(phi, want, rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("act", ["relu", "silu"])
def test_gate_is_a_distribution_and_phi_is_a_convex_combination(act):
    rng = np.random.default_rng(8)
    model, F, gu = small_model(rng, act=act)
    Ff, guf = orc.as_f64(F), orc.as_f64(gu)
    for b in range(3):
        cl = orc.component_logits(Ff[b], model.G, model.logit_scale)
        pi = orc.gating_weights(cl, guf[b], model.gx, model.W1, model.b1, model.W2, model.b2, act)
        assert np.all(pi > 0)
        np.testing.assert_allclose(pi.sum(axis=1), 1.0, rtol=1e-14)
        phi = orc.mol_scores_for(model, Ff[b], guf[b], np.arange(model.G.shape[0]))
        assert np.all(phi >= cl.min(axis=1) - 1e-14) and np.all(phi <= cl.max(axis=1) + 1e-14)


def test_uniform_gate_closed_form():
    """W2 = 0, b2 = 0 => pi = 1/P => phi = <sum_ku f_ku, sum_kx g_kx> * scale / P (from Eq. 6)."""
    rng = np.random.default_rng(9)
    model, F, gu = small_model(rng, scale=3.0)
    model.W2[:] = 0.0
    model.b2[:] = 0.0
    phi = orc.mol_scores(model, F, gu)
    Ff = orc.as_f64(F)
    want = 3.0 * np.einsum("bd,nd->bn", Ff.sum(axis=1), model.G.sum(axis=1)) / model.W2.shape[0]
    np.testing.assert_allclose(phi, want, rtol=1e-12, atol=1e-14)


def test_user_only_gate_reduces_to_weighted_embeddings():
    """If the gate ignores the item and the logits, Eq. 5 holds: the mixture is a sum of dot products
    of pi-weighted user embeddings.  Evaluated here the other way round (weight first, dot after)."""
    rng = np.random.default_rng(10)
    k_u, k_x, d_gu, d_gx = 2, 3, 4, 3
    model, F, gu = small_model(rng, k_u=k_u, k_x=k_x, d_gu=d_gu, d_gx=d_gx, scale=0.7)
    P = k_u * k_x
    model.W1[:, :P] = 0.0                        # no cross input
    model.W1[:, P + d_gu:] = 0.0                 # no item input
    phi = orc.mol_scores(model, F, gu)
    Ff, guf = orc.as_f64(F), orc.as_f64(gu)
    for b in range(3):
        h = np.maximum(model.W1[:, P:P + d_gu] @ guf[b] + model.b1, 0.0)
        z = model.W2 @ h + model.b2
        pi = np.exp(z - z.max())
        pi = (pi / pi.sum()).reshape(k_u, k_x)
        for n in range(model.G.shape[0]):
            want = 0.0
            for kx in range(k_x):
                weighted_user = sum(pi[ku, kx] * Ff[b, ku] for ku in range(k_u))
                want += 0.7 * float(weighted_user @ model.G[n, kx])
            assert abs(phi[b, n] - want) < 1e-12


def test_one_hot_gate_selects_the_indexed_pair():
    """b2 strongly favouring component p* must return <f_{p* div k_x}, g_{p* mod k_x}> * scale."""
    rng = np.random.default_rng(11)
    k_u, k_x = 3, 2
    model, F, gu = small_model(rng, k_u=k_u, k_x=k_x, scale=2.0)
    Ff = orc.as_f64(F)
    for p_star in range(k_u * k_x):
        model.W2[:] = 0.0
        model.b2[:] = 0.0
        model.b2[p_star] = 800.0                 # exp(-800) underflows to exactly 0
        phi = orc.mol_scores(model, F, gu)
        want = 2.0 * np.einsum("bd,nd->bn", Ff[:, p_star // k_x], model.G[:, p_star % k_x])
        np.testing.assert_allclose(phi, want, rtol=1e-13, atol=1e-15)


def test_softmax_shift_invariance():
    rng = np.random.default_rng(12)
    model, F, gu = small_model(rng)
    a = orc.mol_scores(model, F, gu)
    model.b2 += 5.25
    b = orc.mol_scores(model, F, gu)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)


def test_split_first_layer_equals_concatenated():
    """The first gating layer is linear in the concatenation, so it splits exactly into a cross part,
    a user part and an item part (Eq. 8); the item part is what an item-side cache would hold."""
    rng = np.random.default_rng(13)
    model, F, gu = small_model(rng)
    Ff, guf = orc.as_f64(F), orc.as_f64(gu)
    P = model.W2.shape[0]
    d_gu = guf.shape[1]
    item_part = model.gx @ model.W1[:, P + d_gu:].T + model.b1            # cachable
    for b in range(3):
        cl = orc.component_logits(Ff[b], model.G, model.logit_scale)
        user_part = model.W1[:, P:P + d_gu] @ guf[b]
        h = np.maximum(cl @ model.W1[:, :P].T + user_part + item_part, 0.0)
        z = h @ model.W2.T + model.b2
        e = np.exp(z - z.max(axis=1, keepdims=True))
        want = ((e / e.sum(axis=1, keepdims=True)) * cl).sum(axis=1)
        got = orc.mol_scores_for(model, Ff[b], guf[b], np.arange(model.G.shape[0]))
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("act", ["relu", "silu"])
def test_mol_loop_by_loop_rederivation(act):
    """Pure-Python scalar loops over Eq. 3 / Eq. 6 / the 2-layer gate, no numpy broadcasting."""
    import math
    rng = np.random.default_rng(14)
    model, F, gu = small_model(rng, N=6, act=act, scale=1.3)
    Ff, guf = orc.as_f64(F), orc.as_f64(gu)
    k_u, d = Ff.shape[1], Ff.shape[2]
    k_x = model.G.shape[1]
    P, H = k_u * k_x, model.W1.shape[0]
    got = orc.mol_scores(model, F, gu)
    for b in range(3):
        for n in range(6):
            cl = [1.3 * sum(Ff[b, p // k_x, j] * model.G[n, p % k_x, j] for j in range(d)) for p in range(P)]
            x = cl + guf[b].tolist() + model.gx[n].tolist()
            hid = []
            for h in range(H):
                pre = model.b1[h] + sum(model.W1[h, i] * x[i] for i in range(len(x)))
                hid.append(max(pre, 0.0) if act == "relu" else pre / (1.0 + math.exp(-pre)))
            z = [model.b2[p] + sum(model.W2[p, h] * hid[h] for h in range(H)) for p in range(P)]
            m = max(z)
            e = [math.exp(v - m) for v in z]
            phi = sum(ei * ci for ei, ci in zip(e, cl)) / sum(e)
            assert abs(got[b, n] - phi) < 1e-12


def test_negative_candidate_ids_are_padding():
    rng = np.random.default_rng(15)
    model, F, gu = small_model(rng)
    cand = np.array([[3, -1, 7], [0, 1, -1], [-1, -1, 5]])
    sc = orc.mol_scores(model, F, gu, cand)
    full = orc.mol_scores(model, F, gu)
    for b in range(3):
        for j in range(3):
            if cand[b, j] < 0:
                assert sc[b, j] == -np.inf
            else:
                assert sc[b, j] == full[b, cand[b, j]]


# ----------------------------------------------------------------------------- compositions
def _two_stage_case(rng, N=300):
    model, F, gu = small_model(rng, N=N)
    Q1 = rand_bf16_bits(rng, (3, 16))
    X1 = rand_bf16_bits(rng, (N, 16))
    return model, F, gu, Q1, X1


def test_two_stage_with_all_candidates_equals_exhaustive():
    """K' = N is the MoL-only model (Section 5.2.1)."""
    rng = np.random.default_rng(16)
    model, F, gu, Q1, X1 = _two_stage_case(rng)
    a = orc.two_stage(model, Q1, X1, F, gu, Kp=300, k=10)
    e = orc.mol_topk(model, F, gu, None, 10)
    for (ai, asc), (ei, esc) in zip(a, e):
        assert ai.tolist() == ei.tolist() and asc.tolist() == esc.tolist()


def test_two_stage_is_subset_consistent():
    """Every returned item is a stage-1 candidate, and is the best-scored among them."""
    rng = np.random.default_rng(17)
    model, F, gu, Q1, X1 = _two_stage_case(rng)
    res = orc.two_stage(model, Q1, X1, F, gu, Kp=40, k=5)
    s1 = orc.stage1_scores(Q1, X1)
    full = orc.mol_scores(model, F, gu)
    for b, (ids, sc) in enumerate(res):
        cand = sorted(range(300), key=lambda n: (-s1[b, n], n))[:40]
        best = sorted(cand, key=lambda n: (-full[b, n], n))[:5]
        assert ids.tolist() == best


def test_corpus_permutation_invariance():
    rng = np.random.default_rng(18)
    model, F, gu, Q1, X1 = _two_stage_case(rng)
    base = orc.two_stage(model, Q1, X1, F, gu, Kp=50, k=8)
    perm = rng.permutation(300)                            # new row j holds old row perm[j]
    G2 = model.G[perm]
    gx2 = model.gx[perm]
    m2 = orc.MolModel(G2, gx2, model.W1, model.b1, model.W2, model.b2, model.logit_scale, model.act)
    res = orc.two_stage(m2, Q1, X1[perm], F, gu, Kp=50, k=8)
    for (bi, bs), (ri, rs) in zip(base, res):
        assert perm[ri].tolist() == bi.tolist()            # distinct scores: same items, same order
        np.testing.assert_allclose(rs, bs, rtol=1e-12)


def test_batch_split_invariance():
    rng = np.random.default_rng(19)
    model, F, gu, Q1, X1 = _two_stage_case(rng)
    whole = orc.two_stage(model, Q1, X1, F, gu, Kp=50, k=8)
    for b in range(3):
        one = orc.two_stage(model, Q1[b:b + 1], X1, F[b:b + 1], gu[b:b + 1], Kp=50, k=8)[0]
        assert one[0].tolist() == whole[b][0].tolist() and one[1].tolist() == whole[b][1].tolist()
    S = orc.sample_indices(1, 100, 300)
    hw = orc.hindexer(Q1, X1, 30, S)
    for b in range(3):
        h1 = orc.hindexer(Q1[b:b + 1], X1, 30, S)[0]
        assert h1[0].tolist() == hw[b][0].tolist() and h1[2] == hw[b][2]


# --------------------------------------------------------------------------- INT8 stage 1 (Section 4.1.1)
def test_quantize_int8_hand_worked_cases():
    """scale = 2 makes every product exact, so the expected codes follow from round-half-even and the clamp alone."""
    x = np.array([0.0, 0.25, 0.75, 1.25, 1.75, -0.25, -0.75, -1.25, 100.0, -100.0, 63.5, -63.5, 63.75], dtype=np.float32)
    want = np.array([0, 0, 2, 2, 4, 0, -2, -2, 127, -127, 127, -127, 127], dtype=np.int8)
    assert np.array_equal(orc.quantize_int8(x, 2.0), want)
    # the usual scale for unit-range data
    y = np.array([1.0, -1.0, 0.5, -0.5, 0.25], dtype=np.float32)
    assert np.array_equal(orc.quantize_int8(y, 127.0), np.array([127, -127, 64, -64, 32], dtype=np.int8))


def test_quantize_int8_matches_exact_rational_rounding_on_dyadic_scales():
    from fractions import Fraction
    rng = np.random.default_rng(5)
    x32 = rng.normal(size=400).astype(np.float32)
    bits = (x32.view(np.uint32) >> 16).astype(np.uint16)              # truncate to bf16 bit patterns
    for scale in (0.5, 8.0, 64.0):
        got = orc.quantize_int8(bits, scale)
        xs = orc.bf16_bits_to_f64(bits)
        want = [max(-127, min(127, round(Fraction(float(v)) * Fraction(scale)))) for v in xs]   # Fraction.round: half even
        assert got.tolist() == want
        assert np.array_equal(got, orc.quantize_int8(xs.astype(np.float32), scale))               # bf16 bits == fp32 path


def test_quantize_int8_rounds_the_fp32_product_not_the_exact_one():
    """The contract (the library header's: the product x * scale is rounded once to fp32, then halves go to even)
    differs from rounding the exact product when the exact product sits just off a half-integer and its fp32 rounding
    lands on it.  Hand-built fp32 inputs for scale = fp32(311.7) = 0x1.37b334p+8; the exact products are taken with
    rationals, the fp32 ones follow from them by hand: each is within half an fp32 ulp of k + 1/2."""
    from fractions import Fraction
    scale = float(np.float32(311.7))
    assert scale.hex() == "0x1.37b3340000000p+8"
    cases = [
        # (x as fp32 hex, k + 1/2 the fp32 product lands on, code by the contract, code if the exact product were rounded)
        ("-0x1.10ac240000000p-3", -41.5, -42, -41),   # exact magnitude just below 41.5: contract ties to even 42
        ("0x1.58f2720000000p-3", 52.5, 52, 53),       # exact just above 52.5: contract ties to even 52
        ("0x1.71960c0000000p-2", 112.5, 112, 112),    # exact below 112.5, and 112 is the even neighbour: both agree
        ("-0x1.e97f0e0000000p-3", -74.5, -74, -75),   # exact magnitude just above 74.5: contract ties to even 74
    ]
    for xhex, half, by_contract, by_exact in cases:
        x = float.fromhex(xhex)
        assert float(np.float32(x)) == x                                  # the input is an fp32 value
        exact = Fraction(x) * Fraction(scale)
        assert exact != Fraction(half)
        ulp = Fraction(1, 2**(23 - int(np.floor(np.log2(abs(half))))))
        assert abs(exact - Fraction(half)) < ulp / 2                      # so the fp32 product is exactly k + 1/2
        assert round(exact) == by_exact                                   # Fraction.round: nearest, halves to even
        assert round(Fraction(half)) == by_contract
        got = int(orc.quantize_int8(np.array([x], dtype=np.float32), scale)[0])
        assert got == by_contract, (xhex, got)


def test_quantize_int8_is_monotone_and_within_half_a_step():
    rng = np.random.default_rng(6)
    x = np.sort(rng.uniform(-1, 1, size=2000).astype(np.float32))
    q = orc.quantize_int8(x, 127.0).astype(np.int64)
    assert np.all(np.diff(q) >= 0)
    assert np.max(np.abs(q - x.astype(np.float64) * 127.0)) <= 0.5 + 1e-4
    assert q.min() >= -127 and q.max() <= 127


def test_int8_stage1_scores_are_the_integer_dot_products():
    rng = np.random.default_rng(7)
    Q = rng.integers(-127, 128, size=(3, 64), dtype=np.int8)
    X = rng.integers(-127, 128, size=(50, 64), dtype=np.int8)
    X[0] = 127
    Q[0] = 127                                                          # the extreme: 64 * 127 * 127
    s = orc.stage1_scores(Q, X)
    for b in range(3):
        for n in range(50):
            assert s[b, n] == sum(int(Q[b, j]) * int(X[n, j]) for j in range(64))
    assert s[0, 0] == 64 * 127 * 127
    # integer scores tie often: the K' best are taken by (score desc, index asc)
    X[10] = X[20]
    s = orc.stage1_scores(Q, X)
    ids, sc = orc.exact_topk_stage1(Q, X, 50)[1]
    assert list(ids).index(10) + 1 == list(ids).index(20)


# --------------------------------------------------------------------------- Algorithm 1's decomposed gate
def small_decomposed(rng, N=30, k_u=2, k_x=3, d=8, H=5, Hu=4, Hx=6, d_gu=4, d_gx=3, scale=1.0, act="relu"):
    P = k_u * k_x
    G = rand_bf16_bits(rng, (N, k_x, d), 0.5)
    gx = rand_bf16_bits(rng, (N, d_gx), 0.5)

    def mlp(d_in, d_h):
        return (rand_bf16_bits(rng, (d_h, d_in), 0.7), (rng.standard_normal(d_h) * 0.3).astype(np.float32),
                rand_bf16_bits(rng, (P, d_h), 0.7), (rng.standard_normal(P) * 0.3).astype(np.float32))

    model = orc.MolModelDecomposed(G, gx, mlp(d_gu, Hu), mlp(d_gx, Hx), mlp(P, H), logit_scale=scale, act=act)
    F = rand_bf16_bits(rng, (3, k_u, d), 0.5)
    gu = rand_bf16_bits(rng, (3, d_gu), 0.5)
    return model, F, gu


def _with(mlp, Wb=None, bb=None):
    Wa, ba, Wb0, bb0 = mlp
    return (Wa, ba, Wb0 if Wb is None else Wb, bb0 if bb is None else bb)


def test_decomposed_gate_is_a_distribution_and_single_component_is_the_dot_product():
    rng = np.random.default_rng(31)
    model, F, gu = small_decomposed(rng, act="silu", scale=2.0)
    Ff, guf = orc.as_f64(F), orc.as_f64(gu)
    cl = orc.component_logits(Ff[0], model.G, 2.0)
    pi = orc.decomposed_gating(cl, guf[0], model.gx, model.user_mlp, model.item_mlp, model.cross_mlp, "silu")
    assert np.allclose(pi.sum(axis=1), 1.0, atol=1e-14) and np.all(pi > 0)
    phi = orc.mol_scores_for(model, Ff[0], guf[0], np.arange(30))
    assert np.all(phi <= cl.max(axis=1) + 1e-12) and np.all(phi >= cl.min(axis=1) - 1e-12)
    one, F1, gu1 = small_decomposed(rng, k_u=1, k_x=1, scale=0.7)
    s = orc.mol_scores(one, F1, gu1)
    want = 0.7 * np.einsum("bd,nd->bn", orc.as_f64(F1)[:, 0], one.G[:, 0])
    assert np.allclose(s, want, atol=1e-14)


def test_decomposed_gate_all_zero_heads_give_the_mean_logit():
    """Second layers zero: uw = xw = cw = 0, SiLU(0) = 0, so the gate is uniform and phi is the mean component logit."""
    rng = np.random.default_rng(32)
    model, F, gu = small_decomposed(rng)
    P = 6
    Z = lambda m: _with(m, Wb=np.zeros_like(orc.as_f64(m[2])), bb=np.zeros(P))
    model.user_mlp, model.item_mlp, model.cross_mlp = Z(model.user_mlp), Z(model.item_mlp), Z(model.cross_mlp)
    s = orc.mol_scores(model, F, gu)
    Ff = orc.as_f64(F)
    want = np.einsum("bd,nd->bn", Ff.sum(axis=1), model.G.sum(axis=1)) / P
    assert np.allclose(s, want, atol=1e-13)


def test_decomposed_gate_combination_is_a_product_plus_cross_then_silu():
    """Constant heads expose combineFn: uw = a, xw = c (vectors over components), cw = t (scalar shift).
    t -> +large: SiLU is the identity there and the softmax forgets the shift, so pi = softmax(a * c);
    t -> -large: SiLU goes to 0 for every component, so pi is uniform.  A sum instead of a product, a missing SiLU,
    or the SiLU applied after the softmax would each break one of the two limits."""
    rng = np.random.default_rng(33)
    model, F, gu = small_decomposed(rng, N=12)
    P = 6
    a = rng.standard_normal(P)
    c = rng.standard_normal(P)
    zeroW = lambda m: np.zeros_like(orc.as_f64(m[2]))
    model.user_mlp = _with(model.user_mlp, Wb=zeroW(model.user_mlp), bb=a)
    model.item_mlp = _with(model.item_mlp, Wb=zeroW(model.item_mlp), bb=c)
    Ff, guf = orc.as_f64(F), orc.as_f64(gu)
    cl = orc.component_logits(Ff[1], model.G, 1.0)
    e = np.exp(a * c - (a * c).max())
    soft = e / e.sum()
    for t, want in ((60.0, soft), (-60.0, np.full(P, 1.0 / P))):
        model.cross_mlp = _with(model.cross_mlp, Wb=zeroW(model.cross_mlp), bb=np.full(P, t))
        pi = orc.decomposed_gating(cl, guf[1], model.gx, model.user_mlp, model.item_mlp, model.cross_mlp)
        assert np.allclose(pi, want[None, :], atol=1e-12)
        phi = orc.mol_scores_for(model, Ff[1], guf[1], np.arange(12))
        assert np.allclose(phi, cl @ want, atol=1e-12)


def test_decomposed_gate_one_hot_selects_the_user_major_component():
    rng = np.random.default_rng(34)
    model, F, gu = small_decomposed(rng, N=10, k_u=2, k_x=3)
    P = 6
    zeroW = lambda m: np.zeros_like(orc.as_f64(m[2]))
    Ff = orc.as_f64(F)
    for p_star in range(P):
        hot = np.zeros(P)
        hot[p_star] = 200.0
        model.user_mlp = _with(model.user_mlp, Wb=zeroW(model.user_mlp), bb=hot)
        model.item_mlp = _with(model.item_mlp, Wb=zeroW(model.item_mlp), bb=np.ones(P))
        model.cross_mlp = _with(model.cross_mlp, Wb=zeroW(model.cross_mlp), bb=np.zeros(P))
        s = orc.mol_scores(model, F, gu)
        want = np.einsum("bd,nd->bn", Ff[:, p_star // 3], model.G[:, p_star % 3])
        assert np.allclose(s, want, atol=1e-12)


@pytest.mark.parametrize("act", ["relu", "silu"])
def test_decomposed_gate_loop_by_loop(act):
    """Scalar loops over Algorithm 1: three MLPs, product plus cross term, SiLU, softmax, weighted sum."""
    import math
    rng = np.random.default_rng(35)
    model, F, gu = small_decomposed(rng, N=5, act=act, scale=1.7)
    Ff, guf = orc.as_f64(F), orc.as_f64(gu)
    k_u, d = Ff.shape[1], Ff.shape[2]
    k_x = model.G.shape[1]
    P = k_u * k_x
    hidden = (lambda v: max(v, 0.0)) if act == "relu" else (lambda v: v / (1.0 + math.exp(-v)))

    def mlp(m, x):
        Wa, ba, Wb, bb = m
        h = [hidden(ba[i] + sum(Wa[i, j] * x[j] for j in range(len(x)))) for i in range(Wa.shape[0])]
        return [bb[p] + sum(Wb[p, i] * h[i] for i in range(len(h))) for p in range(Wb.shape[0])]

    got = orc.mol_scores(model, F, gu)
    for b in range(3):
        uw = mlp(model.user_mlp, guf[b].tolist())
        for n in range(5):
            cl = [1.7 * sum(Ff[b, p // k_x, j] * model.G[n, p % k_x, j] for j in range(d)) for p in range(P)]
            xw = mlp(model.item_mlp, model.gx[n].tolist())
            cw = mlp(model.cross_mlp, cl)
            z = [uw[p] * xw[p] + cw[p] for p in range(P)]
            z = [v / (1.0 + math.exp(-v)) for v in z]
            m = max(z)
            e = [math.exp(v - m) for v in z]
            phi = sum(ei * ci for ei, ci in zip(e, cl)) / sum(e)
            assert abs(got[b, n] - phi) < 1e-12


def test_gather_items_is_a_row_copy_with_zero_padding():
    rng = np.random.default_rng(41)
    G = rand_bf16_bits(rng, (20, 3, 8), 1.0)
    cand = np.array([[3, 3, -1, 19], [0, -5, 7, 1]])
    out = orc.gather_items(G, cand)
    assert out.shape == (2, 4, 3, 8) and out.dtype == G.dtype
    assert np.array_equal(out[0, 0], G[3]) and np.array_equal(out[0, 1], G[3]) and np.array_equal(out[1, 2], G[7])
    assert not out[0, 2].any() and not out[1, 1].any()
    assert np.array_equal(out[0, 3], G[19]) and np.array_equal(out[1, 0], G[0])


def test_half_precision_inputs_decode_exactly():
    """FP16 inference inputs (Section 4.3) reach the oracle as numpy float16: hand-decoded bit patterns."""
    pat = np.array([0x3C00, 0x3555, 0x0001, 0xFBFF, 0x8000, 0x0400], dtype=np.uint16).view(np.float16)
    want = [1.0, 0.333251953125, 2.0 ** -24, -65504.0, 0.0, 2.0 ** -14]
    assert orc.as_f64(pat).tolist() == want
    # bf16 -> fp16 is exact for the magnitudes the path uses (8 significant bits, exponents well inside half's range)
    rng = np.random.default_rng(51)
    b = rand_bf16_bits(rng, (500,), 1.0)
    v = orc.bf16_bits_to_f64(b)
    v = v[(np.abs(v) > 2.0 ** -14) & (np.abs(v) < 60000)]
    assert np.array_equal(v.astype(np.float16).astype(np.float64), v)


# --------------------------------------------------------------------------- item embeddings generated on the fly (Section 3.1)
def small_generated(rng, N=25, k_u=2, k_c=2, k_g=2, d=8, d_s=5, d_h=6, H=5, d_gu=4, d_gx=3, scale=1.0, act="relu"):
    k_x = k_c + k_g
    P = k_u * k_x
    G = rand_bf16_bits(rng, (N, k_c, d), 0.5)
    gx = rand_bf16_bits(rng, (N, d_gx), 0.5)
    seed = rand_bf16_bits(rng, (N, d_s), 0.7)
    gen = (rand_bf16_bits(rng, (d_h, d_s), 0.7), (rng.standard_normal(d_h) * 0.3).astype(np.float32),
           rand_bf16_bits(rng, (k_g * d, d_h), 0.7), (rng.standard_normal(k_g * d) * 0.3).astype(np.float32))
    W1 = rand_bf16_bits(rng, (H, P + d_gu + d_gx), 0.7)
    W2 = rand_bf16_bits(rng, (P, H), 0.7)
    b1 = (rng.standard_normal(H) * 0.3).astype(np.float32)
    b2 = (rng.standard_normal(P) * 0.3).astype(np.float32)
    F = rand_bf16_bits(rng, (3, k_u, d), 0.5)
    gu = rand_bf16_bits(rng, (3, d_gu), 0.5)
    return dict(G=G, gx=gx, seed=seed, gen=gen, W1=W1, b1=b1, W2=W2, b2=b2, F=F, gu=gu, scale=scale, act=act, k_g=k_g, d=d)


def model_with_explicit_embeddings(m, extra):
    """The cached-path model whose item tensor is m's cached embeddings followed by `extra` [N, k_g, d] (fp64)."""
    G_full = np.concatenate([orc.as_f64(m["G"]), extra], axis=1)
    return orc.MolModel(G_full, m["gx"], m["W1"], m["b1"], m["W2"], m["b2"], m["scale"], m["act"])


def test_generated_embeddings_zero_first_layer_gives_the_normalised_bias():
    """Wa = 0, ba = 0: the hidden layer is act(0) = 0, so every item's generated embeddings are the normalised chunks of
    bb -- the scores must equal the cached path on an item tensor extended by those constant vectors."""
    rng = np.random.default_rng(41)
    m = small_generated(rng)
    Wa, ba, Wb, bb = m["gen"]
    gen = (np.zeros_like(Wa), np.zeros_like(ba), Wb, bb)
    model = orc.MolModel(m["G"], m["gx"], m["W1"], m["b1"], m["W2"], m["b2"], m["scale"], m["act"], seed=m["seed"], gen_mlp=gen)
    const = unit_rows(bb.astype(np.float64).reshape(m["k_g"], m["d"]))
    ref = model_with_explicit_embeddings(m, np.broadcast_to(const, (25, m["k_g"], m["d"])))
    np.testing.assert_allclose(orc.mol_scores(model, m["F"], m["gu"]), orc.mol_scores(ref, m["F"], m["gu"]), rtol=0, atol=1e-12)


def test_generated_embeddings_identity_mlp_returns_the_normalised_seed():
    """d_s = d_h = k_g * d, Wa = Wb = I, zero biases, non-negative seeds, ReLU: e = seed, so the generated embeddings are
    the L2-normalised chunks of the seed."""
    rng = np.random.default_rng(42)
    k_g, d = 2, 8
    m = small_generated(rng, k_g=k_g, d=d, d_s=k_g * d, d_h=k_g * d)
    seed = (np.abs(orc.as_f64(m["seed"])) + 0.125).astype(np.float32)          # non-negative, exactly representable path
    eye = np.eye(k_g * d, dtype=np.float32)
    zero = np.zeros(k_g * d, dtype=np.float32)
    model = orc.MolModel(m["G"], m["gx"], m["W1"], m["b1"], m["W2"], m["b2"], m["scale"], "relu", seed=seed,
                         gen_mlp=(eye, zero, eye, zero))
    extra = unit_rows(seed.astype(np.float64).reshape(25, k_g, d))
    m["act"] = "relu"
    ref = model_with_explicit_embeddings(m, extra)
    np.testing.assert_allclose(orc.mol_scores(model, m["F"], m["gu"]), orc.mol_scores(ref, m["F"], m["gu"]), rtol=0, atol=1e-12)


def test_generated_embeddings_are_unit_vectors_and_ignore_the_output_scale():
    """Eq. 9's normalisation: unit L2 norm per generated embedding; multiplying the output layer (Wb, bb) by a positive
    constant changes nothing (a missing normalisation would scale the logits)."""
    rng = np.random.default_rng(43)
    m = small_generated(rng, act="silu", scale=3.0)
    Wa, ba, Wb, bb = (orc.as_f64(t) for t in m["gen"])
    e = orc.generated_item_embeddings(orc.as_f64(m["seed"]), (Wa, ba, Wb, bb), m["k_g"], m["d"], "silu")
    assert e.shape == (25, m["k_g"], m["d"])
    np.testing.assert_allclose(np.linalg.norm(e, axis=2), 1.0, rtol=0, atol=1e-12)
    e4 = orc.generated_item_embeddings(orc.as_f64(m["seed"]), (Wa, ba, 4.0 * Wb, 4.0 * bb), m["k_g"], m["d"], "silu")
    np.testing.assert_allclose(e4, e, rtol=0, atol=1e-12)
    a = orc.MolModel(m["G"], m["gx"], m["W1"], m["b1"], m["W2"], m["b2"], 3.0, "silu", seed=m["seed"], gen_mlp=(Wa, ba, Wb, bb))
    b = orc.MolModel(m["G"], m["gx"], m["W1"], m["b1"], m["W2"], m["b2"], 3.0, "silu", seed=m["seed"], gen_mlp=(Wa, ba, 4.0 * Wb, 4.0 * bb))
    np.testing.assert_allclose(orc.mol_scores(a, m["F"], m["gu"]), orc.mol_scores(b, m["F"], m["gu"]), rtol=0, atol=1e-12)
    # the generated embeddings take the LAST k_g places of the item-side component order
    cl = orc.component_logits(orc.as_f64(m["F"])[0], np.concatenate([orc.as_f64(m["G"]), e], axis=1), 3.0)
    k_x = 2 + m["k_g"]
    for ku in range(2):
        for j in range(m["k_g"]):
            want = 3.0 * (e[:, j, :] @ orc.as_f64(m["F"])[0, ku])
            np.testing.assert_allclose(cl[:, ku * k_x + 2 + j], want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("act", ["relu", "silu"])
def test_generated_embeddings_loop_by_loop(act):
    import math
    rng = np.random.default_rng(44)
    m = small_generated(rng, N=5, act=act, scale=1.7)
    Wa, ba, Wb, bb = (orc.as_f64(t) for t in m["gen"])
    model = orc.MolModel(m["G"], m["gx"], m["W1"], m["b1"], m["W2"], m["b2"], 1.7, act, seed=m["seed"], gen_mlp=m["gen"])
    got = orc.mol_scores(model, m["F"], m["gu"])
    Ff, guf, Gc, sd = orc.as_f64(m["F"]), orc.as_f64(m["gu"]), orc.as_f64(m["G"]), orc.as_f64(m["seed"])
    k_u, d, k_c, k_g = 2, m["d"], 2, m["k_g"]
    k_x = k_c + k_g
    f_act = (lambda v: max(v, 0.0)) if act == "relu" else (lambda v: v / (1.0 + math.exp(-v)))
    for b in range(3):
        for n in range(5):
            hid = [f_act(ba[u] + sum(Wa[u, i] * sd[n, i] for i in range(sd.shape[1]))) for u in range(Wa.shape[0])]
            e = [bb[f] + sum(Wb[f, u] * hid[u] for u in range(len(hid))) for f in range(k_g * d)]
            rows = [[Gc[n, kx, j] for j in range(d)] for kx in range(k_c)]
            for j in range(k_g):
                chunk = e[j * d:(j + 1) * d]
                nrm = math.sqrt(sum(v * v for v in chunk))
                rows.append([v / nrm for v in chunk])
            cl = [1.7 * sum(Ff[b, p // k_x, j] * rows[p % k_x][j] for j in range(d)) for p in range(k_u * k_x)]
            x = cl + guf[b].tolist() + model.gx[n].tolist()
            h1 = [f_act(model.b1[h] + sum(model.W1[h, i] * x[i] for i in range(len(x)))) for h in range(model.W1.shape[0])]
            z = [model.b2[p] + sum(model.W2[p, h] * h1[h] for h in range(len(h1))) for p in range(len(cl))]
            mz = max(z)
            w = [math.exp(v - mz) for v in z]
            phi = sum(wi * ci for wi, ci in zip(w, cl)) / sum(w)
            assert abs(got[b, n] - phi) < 1e-12
