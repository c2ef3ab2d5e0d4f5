"""One retrieval step (hindexer_topk -> mol_topk, through the C ABI) recorded into a HIP graph and replayed.

Both calls launch kernels only (no memory-set nodes, no allocation, no host synchronisation once the per-process
occupancy queries of the first call are done), so a caller may capture them on its stream.  The graph is replayed
several times with new query contents written into the same buffers and with the program's own eager calls and
synchronisations between the replays; every replay must give what the eager call gives on the same inputs."""
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def m():
    import paper_2306_04039_amd as lib
    return lib


@pytest.mark.parametrize("name,N,B,Kp,lam", [("C2", 300_000, 24, 2048, 0),         # small sample: one selecting kernel
                                             ("C2", 2_000_000, 40, 4096, 131_072),  # large sample: bracket + filtering scan
                                             ("C1", 50_000, 8, 512, 0)])
def test_graph_replays_match_eager(name, N, B, Kp, lam):
    lib = m()
    wl = synth.CONFIGS[name].replace(N=N, B=B, Kp=Kp, bias_scale=0.1)
    cen = synth.make_centres(wl, DEV)
    items, gw = synth.make_items(wl, cen), synth.make_gate_weights(wl, DEV)
    corpus = lib.mol_corpus_pack(items["x1"], items["G"], items["gx"], gw.W1, gw.b1, gw.W2, gw.b2, k_u=wl.k_u,
                                 logit_scale=wl.logit_scale, act=wl.act)
    k = 50
    lam = lam or lib.hindexer_default_lambda(corpus, Kp)
    queries = [synth.make_queries(wl.replace(seed=wl.seed + 17 * r), cen) for r in range(4)]

    def buffers():
        return (torch.empty(lib.hindexer_workspace_bytes(corpus, B, Kp, lam), dtype=torch.uint8, device=DEV),
                torch.empty(lib.mol_workspace_bytes(corpus, B, Kp, k), dtype=torch.uint8, device=DEV),
                (torch.empty(B, Kp, dtype=torch.int32, device=DEV), torch.empty(B, Kp, dtype=torch.float32, device=DEV),
                 torch.empty(B, dtype=torch.int32, device=DEV)),
                (torch.empty(B, k, dtype=torch.int32, device=DEV), torch.empty(B, k, dtype=torch.float32, device=DEV)))

    def step(q1, F, gu, bufs):
        ws1, ws2, o1, o2 = bufs
        lib.hindexer_topk(corpus, q1, Kp, lam=lam, seed=5, workspace=ws1, out=o1)
        lib.mol_topk(corpus, F, gu, o1[0], k, workspace=ws2, out=o2, cand_count=o1[2])

    # the graph's own inputs and outputs
    q1 = queries[0]["q1"].clone()
    F = queries[0]["F"].clone()
    gu = queries[0]["gu"].clone()
    gbufs = buffers()
    step(q1, F, gu, gbufs)  # first call outside the capture: one-time occupancy queries and attribute settings
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(q1, F, gu, gbufs)  # the binding hands torch's current stream, the capturing one, to the library
    torch.cuda.synchronize()

    ebufs = buffers()
    for r in (1, 2, 3, 0, 2):
        q = queries[r]
        # eager result on these queries (own buffers), with a synchronisation before the replay
        step(q["q1"], q["F"], q["gu"], ebufs)
        torch.cuda.synchronize()
        want_idx, want_score, want_count = ebufs[3][0].clone(), ebufs[3][1].clone(), ebufs[2][2].clone()
        q1.copy_(q["q1"])
        F.copy_(q["F"])
        gu.copy_(q["gu"])
        gbufs[3][0].fill_(-5)
        gbufs[3][1].fill_(5.0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(gbufs[2][2], want_count), f"replay for query set {r}: candidate counts differ"
        assert torch.equal(gbufs[3][0], want_idx), f"replay for query set {r}: top-k indices differ"
        assert torch.equal(gbufs[3][1], want_score), f"replay for query set {r}: top-k scores differ"
    corpus.free()
