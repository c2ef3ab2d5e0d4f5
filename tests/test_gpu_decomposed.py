"""GPU parity of Algorithm 1's decomposed gate (user / item / cross MLPs, uw * xw + cw, SiLU, softmax; Section 3.4)."""
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
    "odd-kx8": dict(k_u=2, k_x=8, d_p=32, H=64, d_gu=48, d_gx=16),
    "odd-kx1": dict(k_u=16, k_x=1, d_p=32, H=32, d_gu=32, d_gx=32),
    "odd-h96": dict(k_u=8, k_x=2, d_p=128, H=96, d_gu=20, d_gx=96),
}


def m():
    import paper_2306_04039_amd as lib
    return lib


def build(wl, d_hu=0, d_hx=0):
    cen = synth.make_centres(wl, DEV)
    items = synth.make_items(wl, cen)
    q = synth.make_queries(wl, cen)
    user_mlp, item_mlp, cross_mlp = synth.make_decomposed_gate_weights(wl, DEV, d_hu, d_hx)
    corpus = m().mol_corpus_pack(items["x1"], items["G"], items["gx"], cross_mlp[0], cross_mlp[1], cross_mlp[2], cross_mlp[3],
                                 k_u=wl.k_u, logit_scale=wl.logit_scale, act=wl.act, user_mlp=user_mlp, item_mlp=item_mlp)
    dec = lambda mlp: tuple(bits(t) for t in mlp)
    model = orc.MolModelDecomposed(bits(items["G"]), bits(items["gx"]), dec(user_mlp), dec(item_mlp), dec(cross_mlp),
                                   wl.logit_scale, wl.act)
    return items, q, corpus, model


@pytest.mark.parametrize("shape", list(SHAPES))
@pytest.mark.parametrize("scale,act", [(1.0, "relu"), (20.0, "silu"), (0.05, "relu")])
def test_decomposed_mol_score_matches_oracle(shape, scale, act):
    wl = synth.CONFIGS["C2"].replace(N=3000, B=5, Kp=333, logit_scale=scale, act=act, n_clusters=16, **SHAPES[shape])
    items, q, corpus, model = build(wl, d_hu=48, d_hx=80)
    g = torch.Generator().manual_seed(1)
    cand = torch.stack([torch.randperm(wl.N, generator=g)[:wl.Kp] for _ in range(wl.B)]).to(torch.int32)
    cand[1, 300:] = -1
    got = m().mol_score(corpus, q["F"], q["gu"], cand.to(DEV)).cpu().numpy()
    want = orc.mol_scores(model, bits(q["F"]), bits(q["gu"]), cand.numpy())
    assert np.all(np.isneginf(got[1, 300:]))
    for b in range(wl.B):
        ok = cand[b].numpy() >= 0
        assert_scores_close(got[b][ok], want[b][ok], scale, f"query {b}")
    corpus.free()


def test_decomposed_exhaustive_and_two_stage():
    wl = synth.CONFIGS["C4"].replace(N=20_000, B=6, Kp=1500, k=40, n_clusters=32)
    items, q, corpus, model = build(wl)
    # exhaustive scoring (every item for every query)
    got = m().mol_score(corpus, q["F"], q["gu"]).cpu().numpy()
    want = orc.mol_scores(model, bits(q["F"]), bits(q["gu"]))
    for b in range(wl.B):
        assert_scores_close(got[b], want[b], wl.logit_scale, f"exhaustive, query {b}")
    # the cascade: h-indexer -> decomposed MoL -> top-k
    ci, cs, cc = m().hindexer_topk(corpus, q["q1"], wl.Kp, seed=2)
    idx, sc = m().mol_topk(corpus, q["F"], q["gu"], ci, wl.k)
    torch.cuda.synchronize()
    ci, idx, sc = ci.cpu().numpy(), idx.cpu().numpy(), sc.cpu().numpy()
    for b in range(wl.B):
        cand = ci[b].astype(np.int64)
        lookup = dict(zip(cand.tolist(), want[b][cand].tolist()))
        kth = np.sort(want[b][cand])[::-1][wl.k - 1]
        assert_topk_set(idx[b], lookup, wl.k, 2e-3 * abs(kth) + 1e-4 * wl.logit_scale, f"query {b}")
        assert_scores_close(sc[b], [lookup[i] for i in idx[b].tolist()], wl.logit_scale, f"query {b}")
        assert_sorted_desc(sc[b], idx[b], f"query {b}")
    corpus.free()


def test_decomposed_pack_rejects_missing_weights():
    wl = synth.CONFIGS["C2"].replace(N=100, B=2, n_clusters=4)
    cen = synth.make_centres(wl, DEV)
    items = synth.make_items(wl, cen)
    user_mlp, item_mlp, cross_mlp = synth.make_decomposed_gate_weights(wl, DEV)
    with pytest.raises(ValueError):
        m().mol_corpus_pack(items["x1"], items["G"], items["gx"], *cross_mlp, k_u=wl.k_u, user_mlp=user_mlp)
