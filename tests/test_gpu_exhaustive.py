"""Exhaustive MoL (cand_idx = NULL; Section 5.2.1's MoL-only model, K' = X) at the launch shapes of the large-batch
workload: more than 256 queries (the kernel walks the batch in chunks of 256 per item block) and rows long enough for
the two-level final selection over implicit item indices.  Element by element against the oracle."""
import numpy as np
import pytest
import torch

import synth
from oracle import retrieval_oracle as orc
from parity_util import assert_scores_close, assert_sorted_desc, assert_topk_set, bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

SHAPES = {
    "C1": dict(k_u=4, k_x=4, d_p=32, H=32, d_gu=32, d_gx=32),
    "C2": dict(k_u=4, k_x=4, d_p=64, H=64, d_gu=64, d_gx=64),
    "C3": dict(k_u=8, k_x=4, d_p=64, H=128, d_gu=128, d_gx=128),
    "C4": dict(k_u=8, k_x=8, d_p=64, H=128, d_gu=128, d_gx=128),
    "odd-kx1": dict(k_u=16, k_x=1, d_p=32, H=32, d_gu=32, d_gx=32),
    "odd-h96": dict(k_u=8, k_x=2, d_p=128, H=96, d_gu=20, d_gx=96),
}


def m():
    import paper_2306_04039_amd as lib
    return lib


def build(wl, gate):
    cen = synth.make_centres(wl, DEV)
    items = synth.make_items(wl, cen)
    q = synth.make_queries(wl, cen)
    if gate == "decomposed":
        user_mlp, item_mlp, cross_mlp = synth.make_decomposed_gate_weights(wl, DEV, 48, 80)
        corpus = m().mol_corpus_pack(None, items["G"], items["gx"], *cross_mlp, k_u=wl.k_u, logit_scale=wl.logit_scale,
                                     act=wl.act, user_mlp=user_mlp, item_mlp=item_mlp)
        dec = lambda mlp: tuple(bits(t) for t in mlp)
        model = orc.MolModelDecomposed(bits(items["G"]), bits(items["gx"]), dec(user_mlp), dec(item_mlp), dec(cross_mlp),
                                       wl.logit_scale, wl.act)
    else:
        gw = synth.make_gate_weights(wl, DEV)
        corpus = m().mol_corpus_pack(None, items["G"], items["gx"], gw.W1, gw.b1, gw.W2, gw.b2, k_u=wl.k_u,
                                     logit_scale=wl.logit_scale, act=wl.act)
        model = orc.MolModel(bits(items["G"]), bits(items["gx"]), bits(gw.W1), bits(gw.b1), bits(gw.W2), bits(gw.b2),
                             wl.logit_scale, wl.act)
    return items, q, corpus, model


def checked_queries(B, every):
    """All queries, or the ones around the 256-query chunk boundaries plus a seeded handful."""
    if every:
        return list(range(B))
    edge = {0, 1, B - 1}
    for c in range(256, B, 256):
        edge |= {c - 1, c, c + 1}
    rng = np.random.default_rng(B)
    edge |= set(int(x) for x in rng.integers(0, B, 10))
    return sorted(x for x in edge if 0 <= x < B)


@pytest.mark.parametrize("shape,gate,B,every,act,scale", [
    ("C2", "concat", 300, True, "relu", 1.0),        # every one of the 300 x 20003 scores
    ("C2", "concat", 1024, False, "relu", 1.0),      # the largest batch: four query chunks
    ("C2", "concat", 1023, False, "relu", 20.0),     # sharp gates; the last group of queries is incomplete
    ("C2", "concat", 301, False, "silu", 0.05),      # SiLU takes the general exhaustive kernel
    ("C3", "concat", 258, False, "relu", 1.0),       # two queries per logit product
    ("C1", "concat", 515, False, "relu", 20.0),
    ("odd-kx1", "concat", 300, False, "relu", 1.0),  # one query per logit product
    ("odd-h96", "concat", 270, False, "relu", 1.0),
    ("C4", "concat", 300, False, "relu", 1.0),
    ("C4", "concat", 1024, False, "relu", 1.0),
    ("C2", "decomposed", 300, False, "relu", 1.0),
    ("C4", "decomposed", 1024, False, "relu", 1.0),
])
def test_exhaustive_scores_and_topk_beyond_one_query_chunk(shape, gate, B, every, act, scale):
    N, k = 20_003, 100                              # ragged: the last item block holds 3 items
    wl = synth.CONFIGS["C5"].replace(N=N, B=B, k=k, n_clusters=64, bias_scale=0.1, act=act, logit_scale=scale,
                                     **SHAPES[shape])
    items, q, corpus, model = build(wl, gate)
    got = m().mol_score(corpus, q["F"], q["gu"], None)
    idx, sc = m().mol_topk(corpus, q["F"], q["gu"], None, k)
    torch.cuda.synchronize()
    got, idx, sc = got.cpu().numpy(), idx.cpu().numpy(), sc.cpu().numpy()
    assert got.shape == (B, N) and np.all(np.isfinite(got))
    Fb, gub = bits(q["F"]), bits(q["gu"])
    ids = np.arange(N)
    for b in checked_queries(B, every):
        ref = orc.mol_scores_for(model, orc.as_f64(Fb[b]), orc.as_f64(gub[b]), ids)
        assert_scores_close(got[b], ref, wl.logit_scale, f"{shape}/{gate} B={B} query {b}")
        kth = np.sort(ref)[::-1][k - 1]
        assert_topk_set(idx[b], ref, k, 2e-3 * abs(kth) + 1e-4 * wl.logit_scale, f"query {b}")
    # every query: mol_topk is the exact selection (score desc, index asc) over mol_score's own values
    for b in range(B):
        want = np.lexsort((ids, -got[b].astype(np.float64)))[:k]
        assert idx[b].tolist() == want.tolist(), f"query {b}"
        assert np.array_equal(sc[b], got[b, want])
    # every query: the exhaustive kernel agrees with the per-candidate kernel given the explicit list 0..N-1 (the
    # latter is checked against the oracle element by element in the candidate-list tests)
    sub = list(range(0, B, 37))
    cand = torch.arange(N, dtype=torch.int32, device=DEV).repeat(len(sub), 1)
    via_list = m().mol_score(corpus, q["F"][sub].contiguous(), q["gu"][sub].contiguous(), cand).cpu().numpy()
    assert_scores_close(via_list, got[sub], wl.logit_scale, "exhaustive vs candidate-list kernel")
    corpus.free()


@pytest.mark.parametrize("shift", [300.0, -300.0, 0.0])
def test_exhaustive_softmax_with_gate_logits_outside_the_exponent_range(shift):
    """Gate logits near +-300: without the maximum subtracted their exponentials would leave the fp32 range (inf, or all
    zero).  With shift 0 the biases are spread over +-120 instead: the largest exponential is finite, the others
    underflow against it.  The scores must still be the oracle's."""
    N, B = 5_003, 40
    wl = synth.CONFIGS["C5"].replace(N=N, B=B, k=10, n_clusters=16, bias_scale=0.1, **SHAPES["C2"])
    cen = synth.make_centres(wl, DEV)
    items = synth.make_items(wl, cen)
    q = synth.make_queries(wl, cen)
    gw = synth.make_gate_weights(wl, DEV)
    b2 = gw.b2.clone()
    if shift:
        b2 += shift
    else:
        b2 += torch.linspace(-120.0, 120.0, b2.numel(), device=b2.device)
    corpus = m().mol_corpus_pack(None, items["G"], items["gx"], gw.W1, gw.b1, gw.W2, b2, k_u=wl.k_u,
                                 logit_scale=wl.logit_scale, act=wl.act)
    model = orc.MolModel(bits(items["G"]), bits(items["gx"]), bits(gw.W1), bits(gw.b1), bits(gw.W2), bits(b2),
                         wl.logit_scale, wl.act)
    got = m().mol_score(corpus, q["F"], q["gu"], None).cpu().numpy()
    assert np.all(np.isfinite(got))
    Fb, gub = bits(q["F"]), bits(q["gu"])
    ids = np.arange(N)
    for b in (0, 7, B - 1):
        ref = orc.mol_scores_for(model, orc.as_f64(Fb[b]), orc.as_f64(gub[b]), ids)
        assert_scores_close(got[b], ref, wl.logit_scale, f"shift {shift} query {b}")
    corpus.free()


@pytest.mark.parametrize("N,B,k", [(40_961, 5, 100), (70_000, 260, 10), (300_000, 3, 1024)])
def test_exhaustive_topk_two_level_selection_over_implicit_indices(N, B, k):
    """Rows of >= 16384 x 2 entries take the two-level selection; without a candidate list the item index is the
    position in the row.  Duplicated items put exact ties across slices."""
    wl = synth.CONFIGS["C5"].replace(N=N, B=B, k=k, n_clusters=32, bias_scale=0.1)
    cen = synth.make_centres(wl, DEV)
    items = synth.make_items(wl, cen)
    q = synth.make_queries(wl, cen)
    gw = synth.make_gate_weights(wl, DEV)
    for key in ("G", "gx"):
        items[key][N - 2000:N - 1000] = items[key][0:1000]       # exact duplicates far apart in the row
    corpus = m().mol_corpus_pack(None, items["G"], items["gx"], gw.W1, gw.b1, gw.W2, gw.b2, k_u=wl.k_u,
                                 logit_scale=wl.logit_scale, act=wl.act)
    got = m().mol_score(corpus, q["F"], q["gu"], None)
    idx, sc = m().mol_topk(corpus, q["F"], q["gu"], None, k)
    torch.cuda.synchronize()
    got, idx, sc = got.cpu().numpy(), idx.cpu().numpy(), sc.cpu().numpy()
    assert np.array_equal(got[:, N - 2000:N - 1000], got[:, 0:1000])
    model = orc.MolModel(bits(items["G"]), bits(items["gx"]), bits(gw.W1), bits(gw.b1), bits(gw.W2), bits(gw.b2),
                         wl.logit_scale, wl.act)
    ids = np.arange(N)
    for b in range(B):
        want = np.lexsort((ids, -got[b].astype(np.float64)))[:k]
        assert idx[b].tolist() == want.tolist(), f"query {b}"
        assert np.array_equal(sc[b], got[b, want])
        assert_sorted_desc(sc[b], idx[b], f"query {b}")
    for b in sorted({0, B // 2, B - 1}):
        ref = orc.mol_scores_for(model, orc.as_f64(bits(q["F"])[b]), orc.as_f64(bits(q["gu"])[b]), ids)
        assert_scores_close(got[b], ref, wl.logit_scale, f"query {b}")
        kth = np.sort(ref)[::-1][k - 1]
        assert_topk_set(idx[b], ref, k, 2e-3 * abs(kth) + 1e-4, f"query {b}")
    corpus.free()
