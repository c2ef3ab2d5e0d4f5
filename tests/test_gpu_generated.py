"""GPU parity of item-side embeddings generated on the fly (Section 3.1, item-side bullet): the last k_g of the k_x
item-side embeddings come from a 2-layer MLP on a cached seed, inside the scoring kernel."""
import numpy as np
import pytest
import torch

import synth
from oracle import retrieval_oracle as orc
from parity_util import assert_scores_close, assert_sorted_desc, assert_topk_set, bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
K_G, D_S, D_HG = 2, 32, 64

SHAPES = {
    "C2": dict(k_u=4, k_x=4, d_p=64, H=64, d_gu=64, d_gx=64),
    "C4": dict(k_u=8, k_x=8, d_p=64, H=128, d_gu=128, d_gx=128),
}


def m():
    import paper_2306_04039_amd as lib
    return lib


def build(wl, dtype=torch.bfloat16):
    cen = synth.make_centres(wl, DEV)
    items = synth.make_items(wl, cen)
    q = synth.make_queries(wl, cen)
    gw = synth.make_gate_weights(wl, DEV)
    seed = synth.make_item_seeds(wl, cen, D_S)
    gen = synth.make_gen_mlp(wl, DEV, K_G, D_S, D_HG)
    k_c = wl.k_x - K_G
    G_c = items["G"][:, :k_c].contiguous()                       # the cached embeddings
    conv = (lambda t: t.to(dtype)) if dtype != torch.bfloat16 else (lambda t: t)
    gen16 = (conv(gen[0]), gen[1], conv(gen[2]), gen[3])
    corpus = m().mol_corpus_pack(items["x1"], conv(G_c), conv(items["gx"]), conv(gw.W1), gw.b1, conv(gw.W2), gw.b2, k_u=wl.k_u,
                                 logit_scale=wl.logit_scale, act=wl.act, item_seed=conv(seed), gen_mlp=gen16)
    ob = (lambda t: t.cpu().numpy()) if dtype != torch.bfloat16 else bits
    model = orc.MolModel(ob(conv(G_c)), ob(conv(items["gx"])), ob(conv(gw.W1)), bits(gw.b1), ob(conv(gw.W2)), bits(gw.b2),
                         wl.logit_scale, wl.act, seed=ob(conv(seed)), gen_mlp=(ob(gen16[0]), bits(gen[1]), ob(gen16[2]), bits(gen[3])))
    return items, {k: (conv(v) if k in ("F", "gu") else v) for k, v in q.items()}, corpus, model, ob


@pytest.mark.parametrize("shape", list(SHAPES))
@pytest.mark.parametrize("scale,act", [(1.0, "relu"), (20.0, "relu"), (0.05, "silu")])
def test_generated_embeddings_mol_score_matches_oracle(shape, scale, act):
    N, B, Kp = 9000, 7, 1001
    wl = synth.CONFIGS["C2"].replace(N=N, B=B, Kp=Kp, n_clusters=32, logit_scale=scale, act=act, bias_scale=0.2, **SHAPES[shape])
    items, q, corpus, model, ob = build(wl)
    g = torch.Generator().manual_seed(7)
    cand = torch.randint(0, N, (B, Kp), generator=g, dtype=torch.int32)
    cand[:, :40] = torch.arange(40, dtype=torch.int32)
    cand[1, 5::7] = -1
    cand[2, 900:] = -1
    got = m().mol_score(corpus, q["F"], q["gu"], cand.to(DEV))
    torch.cuda.synchronize()
    ref = orc.mol_scores(model, ob(q["F"]), ob(q["gu"]), cand.numpy())
    assert_scores_close(got.cpu().numpy(), ref, scale, f"{shape} scale={scale} act={act}")
    corpus.free()


def test_generated_embeddings_fp16_corpus():
    wl = synth.CONFIGS["C2"].replace(N=5000, B=5, Kp=700, n_clusters=16, bias_scale=0.2, **SHAPES["C4"])
    items, q, corpus, model, ob = build(wl, torch.float16)
    g = torch.Generator().manual_seed(8)
    cand = torch.randint(0, wl.N, (wl.B, wl.Kp), generator=g, dtype=torch.int32)
    got = m().mol_score(corpus, q["F"], q["gu"], cand.to(DEV))
    torch.cuda.synchronize()
    ref = orc.mol_scores(model, ob(q["F"]), ob(q["gu"]), cand.numpy())
    assert_scores_close(got.cpu().numpy(), ref, 1.0, "fp16 corpus")
    corpus.free()


@pytest.mark.parametrize("shape", list(SHAPES))
def test_generated_embeddings_two_stage_exhaustive_and_gather(shape):
    wl = synth.CONFIGS["C2"].replace(N=30_000, B=6, Kp=1500, k=40, n_clusters=32, bias_scale=0.1, **SHAPES[shape])
    items, q, corpus, model, ob = build(wl)
    # exhaustive scoring over a corpus with generated embeddings (cand_idx = NULL)
    sub = slice(0, 2)
    got = m().mol_score(corpus, q["F"][sub].contiguous(), q["gu"][sub].contiguous(), None).cpu().numpy()
    want = orc.mol_scores(model, ob(q["F"][sub]), ob(q["gu"][sub]))
    assert_scores_close(got, want, wl.logit_scale, "exhaustive")
    # the cascade
    ci, cs, cc = m().hindexer_topk(corpus, q["q1"], wl.Kp, seed=2)
    idx, sc = m().mol_topk(corpus, q["F"], q["gu"], ci, wl.k, cand_count=cc)
    torch.cuda.synchronize()
    ci, idx, sc = ci.cpu().numpy(), idx.cpu().numpy(), sc.cpu().numpy()
    Ff, guf = orc.as_f64(ob(q["F"])), orc.as_f64(ob(q["gu"]))
    for b in range(wl.B):
        phi = orc.mol_scores_for(model, Ff[b], guf[b], ci[b])
        lookup = dict(zip(ci[b].tolist(), phi.tolist()))
        kth = np.sort(phi)[::-1][wl.k - 1]
        assert_topk_set(idx[b], lookup, wl.k, 2e-3 * abs(kth) + 1e-4, f"query {b}")
        assert_scores_close(sc[b], [lookup[i] for i in idx[b].tolist()], wl.logit_scale, f"query {b}")
        assert_sorted_desc(sc[b], idx[b], f"query {b}")
    # index select returns the cached embeddings
    rows = m().gather_items(corpus, torch.from_numpy(ci[:, :50].copy()).to(DEV))
    assert np.array_equal(bits(rows), orc.gather_items(bits(items["G"][:, :wl.k_x - K_G].contiguous()), ci[:, :50]))
    corpus.free()


def test_unsupported_generator_shape_is_rejected():
    wl = synth.CONFIGS["C2"].replace(N=2000, B=2, n_clusters=8, **SHAPES["C2"])
    cen = synth.make_centres(wl, DEV)
    items = synth.make_items(wl, cen)
    gw = synth.make_gate_weights(wl, DEV)
    seed = synth.make_item_seeds(wl, cen, 64)                       # d_s = 64: no instance
    gen = synth.make_gen_mlp(wl, DEV, K_G, 64, D_HG)
    with pytest.raises(m().MolError) as e:
        m().mol_corpus_pack(items["x1"], items["G"][:, :2].contiguous(), items["gx"], gw.W1, gw.b1, gw.W2, gw.b2, k_u=wl.k_u,
                            item_seed=seed, gen_mlp=gen)
    assert e.value.status == -4
