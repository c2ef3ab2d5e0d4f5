"""Cluster-mixture corpus / query generator for the two-stage retrieval workloads.

This module only *draws inputs*.  It holds no dot products against queries, no
top-k, no gating: both the CPU oracle and the HIP library are handed the tensors
produced here (the very same bits) and neither side imports the other.

Recipe (every number is a parameter of `Workload`):
  * C clusters; cluster weights uniform or Zipf(a): w_c ~ (c+1)^-a.
  * one table of unit-norm Gaussian centre directions per tensor kind:
    S[C, d1] (stage-1 vectors), M[C, d_p] (all MoL component embeddings, both
    sides), T[C, d_g] (gate features, both sides).
  * an item (or a query) draws one cluster id z that is shared by all of its
    tensors; each vector is normalise(centre[z] + (sigma/sqrt(dim)) * eps),
    eps ~ N(0, I) drawn independently per vector (per component), i.e. sigma
    is the expected *norm* of the noise.
  * vectors are normalised in fp32 and rounded to bf16 (round-to-nearest-even);
    a stage-1 table declared fp32 stays fp32.
  * gating weights are Xavier-uniform, U(-a, a) with a = sqrt(6/(fan_in+fan_out)),
    rounded to bf16; biases are zero unless `bias_scale` > 0 (parity tests).

Items are generated in fixed chunks of ITEM_CHUNK rows, each chunk from its own
seed, so a 1e8-row corpus can be produced piecewise on the device that will hold
it.  The random stream depends on the torch device type: whoever generates hands
the resulting bits to every consumer.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional, Tuple

import torch

ITEM_CHUNK = 1 << 20
MASTER_SEED = 20230604

# sub-stream tags
_T_CENTRE_S, _T_CENTRE_M, _T_CENTRE_T = 11, 12, 13
_T_W1, _T_W2, _T_B1, _T_B2 = 21, 22, 23, 24
_T_DEC = 50  # decomposed gate: tags 50..61
_T_ITEM, _T_QUERY = 31, 41
_T_SEED, _T_CENTRE_Z, _T_GEN = 35, 14, 70  # seeds of on-the-fly item embeddings, their centre table, the generator MLP


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    N: int
    B: int
    Kp: int                      # stage-1 candidate count K'
    k: int = 100
    d1: int = 64
    stage1_dtype: str = "bf16"   # "bf16" | "f32"
    k_u: int = 4
    k_x: int = 4
    d_p: int = 64
    H: int = 64
    d_gu: int = 64
    d_gx: int = 64
    n_clusters: int = 1024
    zipf_a: float = 0.0          # 0 => uniform cluster weights
    sigma: float = 0.3
    logit_scale: float = 1.0
    act: str = "relu"
    bias_scale: float = 0.0
    seed: int = MASTER_SEED

    @property
    def P(self) -> int:
        return self.k_u * self.k_x

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[str, Workload] = {
    # the five workloads the benchmark contract names, in order
    "C1": Workload("C1-tiny", N=100_000, B=16, Kp=1024, stage1_dtype="f32", k_u=4, k_x=4, d_p=32,
                   H=32, d_gu=32, d_gx=32, n_clusters=256),
    "C2": Workload("C2-1M", N=1_000_000, B=64, Kp=4096, k_u=4, k_x=4, d_p=64, H=64, d_gu=64, d_gx=64,
                   n_clusters=1024),
    "C3": Workload("C3-10M", N=10_000_000, B=128, Kp=16_384, k_u=8, k_x=4, d_p=64, H=128, d_gu=128,
                   d_gx=128, n_clusters=1024, zipf_a=1.1),
    "C4": Workload("C4-100M", N=100_000_000, B=32, Kp=100_000, k_u=8, k_x=8, d_p=64, H=128, d_gu=128,
                   d_gx=128, n_clusters=16_384, zipf_a=1.1),
    "C5": Workload("C5-exhaustive", N=1_000_000, B=1024, Kp=0, k_u=4, k_x=4, d_p=64, H=64, d_gu=64,
                   d_gx=64, n_clusters=1024),
}


@dataclasses.dataclass
class GateWeights:
    W1: torch.Tensor   # bf16 [H, P + d_gu + d_gx]
    b1: torch.Tensor   # f32  [H]
    W2: torch.Tensor   # bf16 [P, H]
    b2: torch.Tensor   # f32  [P]


def _gen(seed: int, tag: int, sub: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1_000_003 + tag * 7_919 + sub * 104_729 + 17) % (2**63 - 1))
    return g


def _unit_rows(x: torch.Tensor) -> torch.Tensor:
    return x / x.norm(dim=-1, keepdim=True).clamp_min(1e-12)


def make_centres(w: Workload, device="cpu") -> Dict[str, torch.Tensor]:
    """Centre tables S, M, T (fp32, unit rows) and the cluster CDF."""
    out = {}
    for key, tag, dim in (("S", _T_CENTRE_S, w.d1), ("M", _T_CENTRE_M, w.d_p), ("T", _T_CENTRE_T, max(w.d_gu, w.d_gx))):
        g = _gen(w.seed, tag, 0, device)
        out[key] = _unit_rows(torch.randn(w.n_clusters, dim, generator=g, device=device, dtype=torch.float32))
    ranks = torch.arange(1, w.n_clusters + 1, device=device, dtype=torch.float64)
    wts = ranks.pow(-w.zipf_a) if w.zipf_a > 0 else torch.ones_like(ranks)
    out["cdf"] = (wts.cumsum(0) / wts.sum()).to(torch.float32)
    return out


def _draw_clusters(n: int, cdf: torch.Tensor, g: torch.Generator) -> torch.Tensor:
    u = torch.rand(n, generator=g, device=cdf.device, dtype=torch.float32)
    return torch.searchsorted(cdf, u).clamp_max(cdf.numel() - 1)


def _noisy_unit(centre_rows: torch.Tensor, reps: int, sigma: float, g: torch.Generator) -> torch.Tensor:
    """centre_rows [n, dim] -> [n, reps, dim] unit vectors with independent noise per rep."""
    n, dim = centre_rows.shape
    eps = torch.randn(n, reps, dim, generator=g, device=centre_rows.device, dtype=torch.float32)
    v = centre_rows[:, None, :] + (sigma / math.sqrt(dim)) * eps
    return _unit_rows(v)


def make_gate_weights(w: Workload, device="cpu") -> GateWeights:
    d_in = w.P + w.d_gu + w.d_gx

    def xavier(rows, cols, tag):
        a = math.sqrt(6.0 / (rows + cols))
        g = _gen(w.seed, tag, 0, device)
        return ((torch.rand(rows, cols, generator=g, device=device, dtype=torch.float32) * 2 - 1) * a).to(torch.bfloat16)

    def bias(n, tag):
        if w.bias_scale <= 0:
            return torch.zeros(n, device=device, dtype=torch.float32)
        g = _gen(w.seed, tag, 0, device)
        return (torch.rand(n, generator=g, device=device, dtype=torch.float32) * 2 - 1) * w.bias_scale

    return GateWeights(W1=xavier(w.H, d_in, _T_W1), b1=bias(w.H, _T_B1), W2=xavier(w.P, w.H, _T_W2), b2=bias(w.P, _T_B2))


def make_decomposed_gate_weights(w: Workload, device="cpu", d_hu: int = 0, d_hx: int = 0, bias_scale: float = 0.1):
    """Weights of the three 2-layer MLPs of the decomposed gate (user, item, cross), Xavier-uniform -> bf16, small uniform
    biases.  Returns (user_mlp, item_mlp, cross_mlp), each (Wa [d_h, d_in], ba [d_h], Wb [P, d_h], bb [P]).
    Hidden widths default to H."""
    d_hu, d_hx = d_hu or w.H, d_hx or w.H

    def mlp(d_in, d_h, tag):
        def xavier(rows, cols, t):
            a = math.sqrt(6.0 / (rows + cols))
            g = _gen(w.seed, t, 0, device)
            return ((torch.rand(rows, cols, generator=g, device=device, dtype=torch.float32) * 2 - 1) * a).to(torch.bfloat16)

        def bias(n, t):
            g = _gen(w.seed, t, 0, device)
            return (torch.rand(n, generator=g, device=device, dtype=torch.float32) * 2 - 1) * bias_scale

        return (xavier(d_h, d_in, tag), bias(d_h, tag + 1), xavier(w.P, d_h, tag + 2), bias(w.P, tag + 3))

    return mlp(w.d_gu, d_hu, _T_DEC), mlp(w.d_gx, d_hx, _T_DEC + 4), mlp(w.P, w.H, _T_DEC + 8)


def item_chunk(w: Workload, centres: Dict[str, torch.Tensor], chunk_id: int,
               want: Tuple[str, ...] = ("x1", "G", "gx")) -> Dict[str, torch.Tensor]:
    """Items [chunk_id*ITEM_CHUNK, min(N, (chunk_id+1)*ITEM_CHUNK)).

    Returns a dict with any of: x1 [n, d1] (bf16 or f32), G [n, k_x, d_p] bf16, gx [n, d_gx] bf16,
    and z [n] int64 (cluster ids).  Tensors not listed in `want` are skipped but the random stream of
    the others is unchanged (each tensor kind has its own generator).
    """
    dev = centres["S"].device
    lo = chunk_id * ITEM_CHUNK
    n = min(w.N, lo + ITEM_CHUNK) - lo
    if n <= 0:
        raise ValueError("chunk_id out of range")
    z = _draw_clusters(n, centres["cdf"], _gen(w.seed, _T_ITEM, 4 * chunk_id + 0, dev))
    out = {"z": z}
    if "x1" in want:
        v = _noisy_unit(centres["S"][z], 1, w.sigma, _gen(w.seed, _T_ITEM, 4 * chunk_id + 1, dev))[:, 0]
        out["x1"] = v if w.stage1_dtype == "f32" else v.to(torch.bfloat16)
    if "G" in want:
        out["G"] = _noisy_unit(centres["M"][z], w.k_x, w.sigma, _gen(w.seed, _T_ITEM, 4 * chunk_id + 2, dev)).to(torch.bfloat16)
    if "gx" in want:
        out["gx"] = _noisy_unit(centres["T"][z][:, : w.d_gx], 1, w.sigma,
                                _gen(w.seed, _T_ITEM, 4 * chunk_id + 3, dev))[:, 0].to(torch.bfloat16)
    return out


def make_items(w: Workload, centres: Dict[str, torch.Tensor], out: Optional[Dict[str, torch.Tensor]] = None,
               progress=None) -> Dict[str, torch.Tensor]:
    """Whole corpus, chunk by chunk, written into preallocated tensors on the centres' device."""
    dev = centres["S"].device
    if out is None:
        out = {
            "x1": torch.empty(w.N, w.d1, device=dev, dtype=torch.float32 if w.stage1_dtype == "f32" else torch.bfloat16),
            "G": torch.empty(w.N, w.k_x, w.d_p, device=dev, dtype=torch.bfloat16),
            "gx": torch.empty(w.N, w.d_gx, device=dev, dtype=torch.bfloat16),
        }
    n_chunks = (w.N + ITEM_CHUNK - 1) // ITEM_CHUNK
    for c in range(n_chunks):
        ch = item_chunk(w, centres, c, want=tuple(k for k in ("x1", "G", "gx") if k in out))
        lo = c * ITEM_CHUNK
        for key in ("x1", "G", "gx"):
            if key in out:
                out[key][lo: lo + ch[key].shape[0]].copy_(ch[key])
        del ch
        if progress is not None:
            progress(c + 1, n_chunks)
    return out


def make_queries(w: Workload, centres: Dict[str, torch.Tensor], B: Optional[int] = None) -> Dict[str, torch.Tensor]:
    """q1 [B, d1] (stage-1 dtype), F [B, k_u, d_p] bf16, gu [B, d_gu] bf16, z [B]."""
    dev = centres["S"].device
    B = w.B if B is None else B
    z = _draw_clusters(B, centres["cdf"], _gen(w.seed, _T_QUERY, 0, dev))
    q1 = _noisy_unit(centres["S"][z], 1, w.sigma, _gen(w.seed, _T_QUERY, 1, dev))[:, 0]
    F = _noisy_unit(centres["M"][z], w.k_u, w.sigma, _gen(w.seed, _T_QUERY, 2, dev)).to(torch.bfloat16)
    gu = _noisy_unit(centres["T"][z][:, : w.d_gu], 1, w.sigma, _gen(w.seed, _T_QUERY, 3, dev))[:, 0].to(torch.bfloat16)
    return {"z": z, "q1": q1 if w.stage1_dtype == "f32" else q1.to(torch.bfloat16), "F": F, "gu": gu}


def make_item_seeds(w: Workload, centres: Dict[str, torch.Tensor], d_s: int) -> torch.Tensor:
    """Seed vectors of the items (the cached input of the MLP that generates item-side embeddings on the fly): bf16
    [N, d_s], noisy unit vectors around a fourth centre table, by the items' cluster ids (re-drawn from the same stream)."""
    dev = centres["S"].device
    Z = _unit_rows(torch.randn(w.n_clusters, d_s, generator=_gen(w.seed, _T_CENTRE_Z, 0, dev), device=dev, dtype=torch.float32))
    out = torch.empty(w.N, d_s, device=dev, dtype=torch.bfloat16)
    n_chunks = (w.N + ITEM_CHUNK - 1) // ITEM_CHUNK
    for c in range(n_chunks):
        lo = c * ITEM_CHUNK
        n = min(w.N, lo + ITEM_CHUNK) - lo
        z = _draw_clusters(n, centres["cdf"], _gen(w.seed, _T_ITEM, 4 * c + 0, dev))
        out[lo: lo + n] = _noisy_unit(Z[z], 1, w.sigma, _gen(w.seed, _T_SEED, c, dev))[:, 0].to(torch.bfloat16)
    return out


def make_gen_mlp(w: Workload, device, k_g: int, d_s: int, d_hg: int, bias_scale: float = 0.1):
    """Weights of the generator MLP (Xavier-uniform -> bf16, small uniform biases): (Wg1 [d_hg, d_s], bg1 [d_hg],
    Wg2 [k_g * d_p, d_hg], bg2 [k_g * d_p])."""
    def xavier(rows, cols, t):
        a = math.sqrt(6.0 / (rows + cols))
        g = _gen(w.seed, t, 0, device)
        return ((torch.rand(rows, cols, generator=g, device=device, dtype=torch.float32) * 2 - 1) * a).to(torch.bfloat16)

    def bias(n, t):
        g = _gen(w.seed, t, 0, device)
        return (torch.rand(n, generator=g, device=device, dtype=torch.float32) * 2 - 1) * bias_scale

    return (xavier(d_hg, d_s, _T_GEN), bias(d_hg, _T_GEN + 1), xavier(k_g * w.d_p, d_hg, _T_GEN + 2), bias(k_g * w.d_p, _T_GEN + 3))
