"""mol_topk_static (the entry point that allocates nothing) against mol_topk, through the C ABI: two calls in a row on
the shared static workspace, the second with a smaller input; plus the size limit and the cand_count argument."""
import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def m():
    import paper_2306_04039_amd as lib
    return lib


def setup(N, B, n_clusters=16):
    wl = synth.CONFIGS["C2"].replace(N=N, B=B, n_clusters=n_clusters, bias_scale=0.1)
    cen = synth.make_centres(wl, DEV)
    items, q, gw = synth.make_items(wl, cen), synth.make_queries(wl, cen), synth.make_gate_weights(wl, DEV)
    corpus = m().mol_corpus_pack(items["x1"], items["G"], items["gx"], gw.W1, gw.b1, gw.W2, gw.b2, k_u=wl.k_u,
                                 logit_scale=wl.logit_scale, act=wl.act)
    return wl, q, corpus


def both(corpus, q, cand, k, B, cand_count=None):
    F, gu = q["F"][:B].contiguous(), q["gu"][:B].contiguous()
    ref = m().mol_topk(corpus, F, gu, cand, k, cand_count=cand_count)
    out = (torch.full((B, k), -7, dtype=torch.int32, device=DEV), torch.full((B, k), 7.0, dtype=torch.float32, device=DEV))
    got = m().mol_topk_static(corpus, F, gu, cand, k, out, cand_count=cand_count)
    torch.cuda.synchronize()
    return ref, got


def test_static_workspace_matches_mol_topk_on_two_calls_in_a_row():
    wl, q, corpus = setup(60_000, 12)
    g = torch.Generator().manual_seed(3)
    # first call: rows of 40000 (two-level selection, ~2 MB of scores in the static workspace)
    big = torch.stack([torch.randperm(wl.N, generator=g)[:40_000] for _ in range(12)]).to(torch.int32)
    big[3, 100::9] = -1
    ref, got = both(corpus, q, big.to(DEV), 100, 12)
    assert torch.equal(ref[0], got[0]) and torch.equal(ref[1], got[1])
    assert int(got[0].min()) >= 0
    # second call, smaller in every dimension: whatever the first left in the workspace must not show
    small = torch.stack([torch.randperm(wl.N, generator=g)[:777] for _ in range(5)]).to(torch.int32)
    small[1, 500:] = -1
    ref2, got2 = both(corpus, q, small.to(DEV), 20, 5)
    assert torch.equal(ref2[0], got2[0]) and torch.equal(ref2[1], got2[1])
    # and the exhaustive form (cand_idx = NULL) on the same workspace: 5 x 60000 scores
    ref3, got3 = both(corpus, q, None, 50, 5)
    assert torch.equal(ref3[0], got3[0]) and torch.equal(ref3[1], got3[1])
    corpus.free()


def test_static_workspace_with_cand_count_and_size_limit():
    lib = m()
    wl, q, corpus = setup(30_000, 6)
    g = torch.Generator().manual_seed(4)
    cand = torch.stack([torch.randperm(wl.N, generator=g)[:3000] for _ in range(6)]).to(torch.int32)
    counts = torch.tensor([3000, 0, 1, 1500, 2999, 64], dtype=torch.int32)
    padded = cand.clone()
    for b in range(6):
        padded[b, counts[b]:] = -1
    # with cand_count, the slots past the count may hold anything: same result as the padded rows without it
    ref, got = both(corpus, q, cand.to(DEV), 100, 6, cand_count=counts.to(DEV))
    want = lib.mol_topk(corpus, q["F"][:6].contiguous(), q["gu"][:6].contiguous(), padded.to(DEV), 100)
    torch.cuda.synchronize()
    for a in (ref, got):
        assert torch.equal(a[0], want[0]) and torch.equal(a[1], want[1])
    assert int((got[0][1] >= 0).sum()) == 0 and int((got[0][2] >= 0).sum()) == 1
    # beyond the static maximum: rejected, outputs untouched
    limit = lib.topk_static_max_bytes()
    Kp_big = limit // (4 * 6) + 1024
    assert lib.mol_workspace_bytes(corpus, 6, Kp_big, 100) > limit
    too_big = torch.zeros(6, Kp_big, dtype=torch.int32, device=DEV)
    out = (torch.full((6, 100), -7, dtype=torch.int32, device=DEV), torch.full((6, 100), 7.0, dtype=torch.float32, device=DEV))
    with pytest.raises(lib.MolError) as e:
        lib.mol_topk_static(corpus, q["F"][:6].contiguous(), q["gu"][:6].contiguous(), too_big, 100, out)
    assert e.value.status == -3
    assert int(out[0].min()) == -7 and float(out[1].max()) == 7.0
    corpus.free()
