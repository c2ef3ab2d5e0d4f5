"""GPU parity of the INT8 stage 1 (Section 4.1.1): integer work, so everything is compared bit for bit."""
import numpy as np
import pytest
import torch

import synth
from oracle import retrieval_oracle as orc
from parity_util import bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FORCE_REDO = 0x100


def m():
    import paper_2306_04039_amd as lib
    return lib


def quantised(wl, scale_x=None, scale_q=None):
    """bf16 workload tensors -> int8 on the GPU (library) and on the CPU (oracle), each with its own code."""
    cen = synth.make_centres(wl, DEV)
    items = synth.make_items(wl, cen)
    q = synth.make_queries(wl, cen)
    gw = synth.make_gate_weights(wl, DEV)
    sx = scale_x or 127.0 / float(items["x1"].float().abs().max())
    sq = scale_q or 127.0 / float(q["q1"].float().abs().max())
    x8 = m().quantize_int8(items["x1"], sx)
    q8 = m().quantize_int8(q["q1"], sq)
    torch.cuda.synchronize()
    x8_o = orc.quantize_int8(bits(items["x1"]), sx)
    q8_o = orc.quantize_int8(bits(q["q1"]), sq)
    return items, q, gw, x8, q8, x8_o, q8_o


@pytest.mark.parametrize("dtype,shape,scale", [("bf16", (1000, 64), 127.0), ("bf16", (777, 64), 311.7), ("f32", (123, 64), 90.5),
                                               ("f32", (3,), 2.0), ("bf16", (8,), 0.25)])
def test_quantize_int8_bit_exact(dtype, shape, scale):
    g = torch.Generator(device=DEV).manual_seed(3)
    x = torch.randn(*shape, generator=g, device=DEV) * 0.4
    x = x.to(torch.bfloat16) if dtype == "bf16" else x
    got = m().quantize_int8(x, scale).cpu().numpy()
    want = orc.quantize_int8(bits(x), scale)
    assert got.dtype == np.int8 and np.array_equal(got, want)


def test_quantize_int8_ties_and_clamp():
    x = torch.tensor([0.0, 0.25, 0.75, 1.25, 1.75, -0.25, -0.75, -1.25, 100.0, -100.0, 63.5, -63.5, 63.75, 3.0, 5.0, 7.0],
                     dtype=torch.float32, device=DEV)
    got = m().quantize_int8(x, 2.0).cpu().numpy().tolist()
    assert got == [0, 0, 2, 2, 4, 0, -2, -2, 127, -127, 127, -127, 127, 6, 10, 14]


def check_exact(ci, cs, cc, s, Kp, what):
    """Integer scores: the K' best under (score desc, index asc) are unique, so sets and scores must match exactly."""
    ci, cs, cc = ci.cpu().numpy(), cs.cpu().numpy(), cc.cpu().numpy()
    assert np.all(cc == Kp), f"{what}: counts {cc}"
    for b in range(s.shape[0]):
        ids, sc = orc.topk_desc(s[b], Kp)
        assert np.array_equal(np.sort(ci[b]), np.sort(ids)), f"{what}: query {b} candidate set differs"
        assert np.array_equal(cs[b].astype(np.float64), s[b, ci[b]]), f"{what}: query {b} scores differ"


@pytest.mark.parametrize("N,B,Kp", [(50_003, 20, 512), (40_001, 16, 1024), (70_000, 70, 300), (3_000, 5, 900)])
def test_hindexer_int8_exact_topk(N, B, Kp):
    wl = synth.CONFIGS["C2"].replace(N=N, B=B, Kp=Kp, n_clusters=64)
    items, q, gw, x8, q8, x8_o, q8_o = quantised(wl)
    assert np.array_equal(x8.cpu().numpy(), x8_o) and np.array_equal(q8.cpu().numpy(), q8_o)
    corpus = m().mol_corpus_pack(x8, items["G"], items["gx"], gw.W1, gw.b1, gw.W2, gw.b2, k_u=wl.k_u)
    s = orc.stage1_scores(q8_o, x8_o)
    assert s.dtype == np.float64 and np.all(s == np.rint(s))
    out = m().hindexer_topk(corpus, q8, Kp, seed=9)
    torch.cuda.synchronize()
    check_exact(*out, s, Kp, "sampled threshold")
    out = m().hindexer_topk(corpus, q8, Kp, seed=9, mode=m().HINDEXER_EXACT | FORCE_REDO)
    torch.cuda.synchronize()
    check_exact(*out, s, Kp, "forced exact redo")
    corpus.free()


def test_hindexer_int8_paper_mode_is_algorithm_2():
    wl = synth.CONFIGS["C2"].replace(N=60_000, B=12, Kp=1000, n_clusters=64)
    items, q, gw, x8, q8, x8_o, q8_o = quantised(wl)
    corpus = m().mol_corpus_pack(x8, items["G"], items["gx"], gw.W1, gw.b1, gw.W2, gw.b2, k_u=wl.k_u)
    lam = 6000
    seed = 77
    ci, cs, cc = m().hindexer_topk(corpus, q8, wl.Kp, lam=lam, seed=seed, mode=m().HINDEXER_PAPER)
    torch.cuda.synchronize()
    S = orc.sample_indices(seed, lam, wl.N)
    ref = orc.hindexer(q8_o, x8_o, wl.Kp, S)
    ci, cs, cc = ci.cpu().numpy(), cs.cpu().numpy(), cc.cpu().numpy()
    for b in range(wl.B):
        ids, sc, t = ref[b]
        assert cc[b] == len(ids)
        assert np.array_equal(np.sort(ci[b, :cc[b]]), np.sort(ids))
        assert np.all(ci[b, cc[b]:] == -1)


def test_two_stage_with_int8_stage1_matches_oracle_cascade():
    """INT8 stage 1 -> MoL -> top-k, against the oracle run on the oracle's own quantised table."""
    from parity_util import assert_scores_close, assert_sorted_desc, assert_topk_set
    wl = synth.CONFIGS["C2"].replace(N=30_000, B=6, Kp=700, k=50, n_clusters=64)
    items, q, gw, x8, q8, x8_o, q8_o = quantised(wl)
    corpus = m().mol_corpus_pack(x8, items["G"], items["gx"], gw.W1, gw.b1, gw.W2, gw.b2, k_u=wl.k_u,
                                 logit_scale=wl.logit_scale, act=wl.act)
    ci, cs, cc = m().hindexer_topk(corpus, q8, wl.Kp, seed=1)
    idx, sc = m().mol_topk(corpus, q["F"], q["gu"], ci, wl.k)
    torch.cuda.synchronize()
    model = orc.MolModel(bits(items["G"]), bits(items["gx"]), bits(gw.W1), bits(gw.b1), bits(gw.W2), bits(gw.b2),
                         wl.logit_scale, wl.act)
    s = orc.stage1_scores(q8_o, x8_o)
    idx, sc = idx.cpu().numpy(), sc.cpu().numpy()
    for b in range(wl.B):
        cand, _ = orc.topk_desc(s[b], wl.Kp)
        phi = orc.mol_scores_for(model, orc.as_f64(bits(q["F"])[b]), orc.as_f64(bits(q["gu"])[b]), cand)
        lookup = dict(zip(cand.tolist(), phi.tolist()))
        kth = np.sort(phi)[::-1][wl.k - 1]
        assert_topk_set(idx[b], lookup, wl.k, 2e-3 * abs(kth) + 1e-4 * wl.logit_scale, f"query {b}")
        assert_scores_close(sc[b], [lookup[i] for i in idx[b].tolist()], wl.logit_scale, f"query {b}")
        assert_sorted_desc(sc[b], idx[b], f"query {b}")
    corpus.free()
