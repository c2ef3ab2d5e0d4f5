"""GPU edge cases: smallest and largest sizes the boundary accepts, and the two-level final selection with ties and padding."""
import numpy as np
import pytest
import torch

import synth
from oracle import retrieval_oracle as orc
from parity_util import assert_scores_close, assert_sorted_desc, assert_topk_set, bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
S1_TOL = 2e-6


def m():
    import paper_2306_04039_amd as lib
    return lib


def make(wl):
    cen = synth.make_centres(wl, DEV)
    return synth.make_items(wl, cen), synth.make_queries(wl, cen), synth.make_gate_weights(wl, DEV)


def pack(wl, items, gw):
    return m().mol_corpus_pack(items["x1"], items["G"], items["gx"], gw.W1, gw.b1, gw.W2, gw.b2, k_u=wl.k_u,
                               logit_scale=wl.logit_scale, act=wl.act)


def check_two_stage(wl, items, q, gw, corpus, queries):
    ci, cs, cc = m().hindexer_topk(corpus, q["q1"], wl.Kp, seed=3)
    idx, sc = m().mol_topk(corpus, q["F"], q["gu"], ci, wl.k)
    torch.cuda.synchronize()
    s = orc.stage1_scores(bits(q["q1"]), bits(items["x1"]))
    model = orc.MolModel(bits(items["G"]), bits(items["gx"]), bits(gw.W1), bits(gw.b1), bits(gw.W2), bits(gw.b2),
                         wl.logit_scale, wl.act)
    ci, cc, idx, sc = ci.cpu().numpy(), cc.cpu().numpy(), idx.cpu().numpy(), sc.cpu().numpy()
    kp_eff = min(wl.Kp, wl.N)
    assert np.all(cc == kp_eff)
    for b in queries:
        assert_topk_set(ci[b, :kp_eff], s[b], kp_eff, S1_TOL, f"stage 1, query {b}")
        cand = ci[b, :kp_eff].astype(np.int64)
        phi = orc.mol_scores_for(model, orc.as_f64(bits(q["F"])[b]), orc.as_f64(bits(q["gu"])[b]), cand)
        lookup = dict(zip(cand.tolist(), phi.tolist()))
        kk = min(wl.k, kp_eff)
        kth = np.sort(phi)[::-1][kk - 1]
        assert_topk_set(idx[b, :kk], lookup, kk, 2e-3 * abs(kth) + 1e-4 * wl.logit_scale, f"stage 2, query {b}")
        assert_scores_close(sc[b, :kk], [lookup[i] for i in idx[b, :kk].tolist()], wl.logit_scale, f"query {b}")
        assert_sorted_desc(sc[b, :kk], idx[b, :kk], f"query {b}")
        assert np.all(idx[b, kk:] == -1) and np.all(np.isneginf(sc[b, kk:]))


@pytest.mark.parametrize("N,B,Kp,k", [(1, 1, 1, 1), (17, 2, 17, 5), (31, 3, 1, 1), (33, 1, 20, 20), (64, 4, 64, 100)])
def test_tiny_corpora(N, B, Kp, k):
    wl = synth.CONFIGS["C2"].replace(N=N, B=B, Kp=Kp, k=k, n_clusters=min(4, N))
    items, q, gw = make(wl)
    corpus = pack(wl, items, gw)
    check_two_stage(wl, items, q, gw, corpus, range(B))
    corpus.free()


def test_largest_batch():
    """B = 1024 is the largest batch the boundary takes (eight launches of 128 queries in the scan)."""
    wl = synth.CONFIGS["C1"].replace(N=6000, B=1024, Kp=64, k=8, n_clusters=16)
    items, q, gw = make(wl)
    corpus = pack(wl, items, gw)
    check_two_stage(wl, items, q, gw, corpus, [0, 1, 127, 128, 500, 1023])
    with pytest.raises(m().MolError) as e:
        m().hindexer_topk(corpus, torch.cat([q["q1"], q["q1"][:1]]), wl.Kp)
    assert e.value.status == -1
    corpus.free()


@pytest.mark.parametrize("Kp,k", [(4000, 1024), (40_000, 1024), (20_000, 100), (20_000, 7), (8192, 1)])
def test_final_selection_levels_with_ties_and_padding(Kp, k):
    """Single-level (k large against the row) and two-level selection give the k best under (score desc, index asc),
    with duplicated items (exact ties across slices) and padding scattered through the candidate rows."""
    wl = synth.CONFIGS["C2"].replace(N=50_000, B=3, n_clusters=8)
    items, q, gw = make(wl)
    for key in ("G", "gx"):
        items[key][25_000:26_000] = items[key][0:1000]           # 1000 exact duplicates, far apart in the row
    corpus = pack(wl, items, gw)
    g = torch.Generator().manual_seed(Kp + k)
    cand = torch.stack([torch.randperm(wl.N, generator=g)[:Kp] for _ in range(3)]).to(torch.int32)
    cand[0, :1000] = torch.arange(1000, dtype=torch.int32)
    cand[0, Kp - 1000:] = torch.arange(25_000, 26_000, dtype=torch.int32)
    cand[1, torch.rand(Kp, generator=g) < 0.3] = -1              # 30 % padding anywhere
    cand[2, k // 2:] = -1                                        # fewer valid candidates than k
    idx, sc = m().mol_topk(corpus, q["F"], q["gu"], cand.to(DEV), k)
    scores = m().mol_score(corpus, q["F"], q["gu"], cand.to(DEV)).cpu().numpy()
    idx, sc = idx.cpu().numpy(), sc.cpu().numpy()
    for b in range(3):
        ids = cand[b].numpy()
        valid = ids >= 0
        ids_v, s_v = ids[valid], scores[b][valid].astype(np.float64)
        assert np.all(np.isneginf(scores[b][~valid]))
        # row 0 lists some items twice (the overwritten head and tail can repeat a random pick): keep one copy each
        ids_u, first = np.unique(ids_v, return_index=True)
        if b != 0:
            assert len(ids_u) == len(ids_v)
        kk = min(k, len(ids_v))
        want = np.lexsort((ids_v, -s_v))[:kk]
        assert idx[b, :kk].tolist() == ids_v[want].tolist(), f"row {b}"
        assert np.array_equal(sc[b, :kk], scores[b][valid][want])
        assert np.all(idx[b, kk:] == -1) and np.all(np.isneginf(sc[b, kk:]))
    corpus.free()


@pytest.mark.parametrize("Kp,k", [(20_000, 64), (20_000, 100), (30_000, 394), (60_000, 64), (3000, 1024)])
def test_final_selection_with_items_listed_more_than_once(Kp, k):
    """Candidate rows drawn with replacement from a small corpus: most items appear several times, so copies of the k-th
    element itself compete for the last places (in a slice of the two-level form, and in the final selection).  Every
    entry that comes before the k-th must be returned, and copies of the k-th fill the rest: the result is the first k
    of the row's entries sorted by (score descending, index ascending), copies included."""
    wl = synth.CONFIGS["C2"].replace(N=4000, B=5, n_clusters=8)
    items, q, gw = make(wl)
    corpus = pack(wl, items, gw)
    g = torch.Generator().manual_seed(Kp + k)
    cand = torch.randint(0, wl.N, (wl.B, Kp), generator=g, dtype=torch.int32)
    cand[1, torch.rand(Kp, generator=g) < 0.5] = -1
    cand = cand.to(DEV)
    idx, sc = m().mol_topk(corpus, q["F"], q["gu"], cand, k)
    scores = m().mol_score(corpus, q["F"], q["gu"], cand).cpu().numpy()
    idx, sc, ids = idx.cpu().numpy(), sc.cpu().numpy(), cand.cpu().numpy()
    for b in range(wl.B):
        valid = ids[b] >= 0
        ids_v, s_v = ids[b][valid], scores[b][valid]
        want = np.lexsort((ids_v, -s_v.astype(np.float64)))[:k]
        assert idx[b].tolist() == ids_v[want].tolist(), f"row {b}"
        assert np.array_equal(sc[b], s_v[want])
    corpus.free()


@pytest.mark.parametrize("Kp", [20_000, 60_000])
def test_final_selection_of_a_row_sorted_by_score(Kp):
    """Candidate rows in ascending and in descending score order.  The bound taken from the head of an ascending row (or
    slice) lets everything through, so the collecting pass overflows its buffer and the multi-pass selection takes over;
    the head of a descending row gives the final bound at once.  Both must return the exact top-k."""
    k = 100
    wl = synth.CONFIGS["C2"].replace(N=80_000, B=2, n_clusters=8)
    items, q, gw = make(wl)
    corpus = pack(wl, items, gw)
    g = torch.Generator().manual_seed(Kp)
    pick = torch.randperm(wl.N, generator=g)[:Kp].to(torch.int32)
    cand = torch.stack([pick, pick]).to(DEV)
    scores = m().mol_score(corpus, q["F"], q["gu"], cand)
    order = torch.argsort(scores, dim=1)                       # ascending
    cand = torch.gather(cand, 1, order.to(torch.int64))
    cand[1] = torch.flip(cand[1], dims=[0])                    # row 1 descending
    cand = cand.contiguous()
    idx, sc = m().mol_topk(corpus, q["F"], q["gu"], cand, k)
    scores = m().mol_score(corpus, q["F"], q["gu"], cand).cpu().numpy()
    idx, sc, ids = idx.cpu().numpy(), sc.cpu().numpy(), cand.cpu().numpy()
    for b in range(2):
        want = np.lexsort((ids[b], -scores[b].astype(np.float64)))[:k]
        assert idx[b].tolist() == ids[b][want].tolist(), f"row {b}"
        assert np.array_equal(sc[b], scores[b][want])
    corpus.free()


@pytest.mark.parametrize("shape", [dict(k_u=16, k_x=1, d_p=32, H=32, d_gu=32, d_gx=32), dict(k_u=8, k_x=8, d_p=64, H=128, d_gu=128, d_gx=128)])
def test_gather_items_is_a_bit_exact_row_copy(shape):
    """Index select (Section 4.1.3): rows of 64 B and of 1 KB, with padding and repeated ids."""
    wl = synth.CONFIGS["C2"].replace(N=5000, B=4, n_clusters=8, **shape)
    items, q, gw = make(wl)
    corpus = pack(wl, items, gw)
    g = torch.Generator().manual_seed(5)
    cand = torch.randint(0, wl.N, (4, 777), generator=g).to(torch.int32)
    cand[0, ::7] = -1
    cand[1, :] = 4999
    cand[2, 100:] = -1
    got = m().gather_items(corpus, cand.to(DEV))
    torch.cuda.synchronize()
    want = orc.gather_items(bits(items["G"]), cand.numpy())
    assert np.array_equal(bits(got), want)
    # timing-free sanity of the error path
    with pytest.raises(m().MolError):
        m().load_library()
        from paper_2306_04039_amd import binding
        binding._check(binding.load_library().mol_gather_items(corpus.handle, None, 4, 777, None, None))
    corpus.free()


@pytest.mark.parametrize("shape", [dict(k_u=8, k_x=8, d_p=64, H=128, d_gu=128, d_gx=128), dict(k_u=4, k_x=4, d_p=64, H=64, d_gu=64, d_gx=64)])
def test_scores_do_not_depend_on_launch_size(shape):
    """The same (query, item) pairs scored alone (a handful of wavefronts on the whole chip) and inside a large call must
    agree bit for bit, and so must the stage-1 scores of a tiny and a large scan: results may not depend on how busy the
    compute units are (matrix-core results read too early would show up here)."""
    wl = synth.CONFIGS["C2"].replace(N=60_000, B=8, n_clusters=16, **shape)
    items, q, gw = make(wl)
    corpus = pack(wl, items, gw)
    g = torch.Generator().manual_seed(9)
    big = torch.stack([torch.randperm(wl.N, generator=g)[:20_000] for _ in range(8)]).to(torch.int32).to(DEV)
    s_big = m().mol_score(corpus, q["F"], q["gu"], big)
    for b in (0, 5):
        for lo, n in ((0, 64), (777, 33), (19_000, 1000)):
            small = big[b:b + 1, lo:lo + n].contiguous()
            s_small = m().mol_score(corpus, q["F"][b:b + 1], q["gu"][b:b + 1], small)
            assert torch.equal(s_small[0], s_big[b, lo:lo + n]), (b, lo, n)
    # stage 1: every score of the full corpus (K' = N: one big scan) vs the scan of a 64-item slice of it (one wavefront busy)
    ci, cs, cc = m().hindexer_topk(corpus, q["q1"], wl.N)
    small_corpus = m().mol_corpus_pack(items["x1"][:64].contiguous(), items["G"][:64].contiguous(), items["gx"][:64].contiguous(),
                                       gw.W1, gw.b1, gw.W2, gw.b2, k_u=wl.k_u)
    ci2, cs2, cc2 = m().hindexer_topk(small_corpus, q["q1"], 64)
    torch.cuda.synchronize()
    for b in range(8):
        full = dict(zip(ci[b].tolist(), cs[b].tolist()))
        part = dict(zip(ci2[b].tolist(), cs2[b].tolist()))
        assert sorted(part) == list(range(64)) and len(full) == wl.N
        assert all(part[i] == full[i] for i in part)
    small_corpus.free()
    corpus.free()
