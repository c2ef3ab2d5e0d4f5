"""The input generator: shapes, dtypes, determinism and the structure the workloads call for."""
import torch

import synth


def test_tiny_workload_shapes_and_norms():
    w = synth.CONFIGS["C1"].replace(N=5000)
    c = synth.make_centres(w)
    items = synth.make_items(w, c)
    q = synth.make_queries(w, c)
    assert items["x1"].shape == (5000, 64) and items["x1"].dtype == torch.float32
    assert items["G"].shape == (5000, 4, 32) and items["G"].dtype == torch.bfloat16
    assert items["gx"].shape == (5000, 32) and items["gx"].dtype == torch.bfloat16
    assert q["q1"].shape == (16, 64) and q["F"].shape == (16, 4, 32) and q["gu"].shape == (16, 32)
    assert torch.allclose(items["x1"].norm(dim=-1), torch.ones(5000), atol=1e-5)
    assert torch.allclose(items["G"].float().norm(dim=-1), torch.ones(5000, 4), atol=2e-2)   # bf16 rounding
    gw = synth.make_gate_weights(w)
    assert gw.W1.shape == (32, 16 + 32 + 32) and gw.W2.shape == (16, 32)
    assert gw.W1.dtype == torch.bfloat16 and float(gw.b1.abs().max()) == 0.0
    a = (6.0 / (32 + 80)) ** 0.5
    assert float(gw.W1.float().abs().max()) <= a * 1.01


def test_generation_is_deterministic_and_clustered():
    w = synth.CONFIGS["C2"].replace(N=3000, n_clusters=16)
    c = synth.make_centres(w)
    a = synth.item_chunk(w, c, 0)
    b = synth.item_chunk(w, c, 0, want=("G",))
    assert torch.equal(a["G"], b["G"]) and torch.equal(a["z"], b["z"])
    # same-cluster stage-1 vectors are close to 1/(1+sigma^2) in cosine, others near 0
    x = a["x1"].float()
    z = a["z"]
    cos = x @ x.T
    same = z[:, None] == z[None, :]
    assert float(cos[same].mean()) > 0.85 and abs(float(cos[~same].mean())) < 0.1


def test_zipf_weights_make_a_head_cluster():
    w = synth.CONFIGS["C4"].replace(N=20000)
    c = synth.make_centres(w)
    z = synth.item_chunk(w, c, 0, want=())["z"]
    share = float((z == 0).float().mean())
    assert 0.10 < share < 0.20
