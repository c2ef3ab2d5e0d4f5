"""Shared helpers for the GPU parity tests: bit-exact hand-over of tensors to the oracle and
tolerance-aware comparison of top-k sets (fp32 on the GPU, fp64 in the oracle)."""
import numpy as np
import torch

RTOL = 2e-3        # relative tolerance on MoL scores
ATOL_UNIT = 1e-4   # absolute floor, multiplied by logit_scale


def bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> uint16 bit patterns (what the oracle decodes itself); fp32 -> float32 array."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def assert_topk_set(gpu_ids, oracle_scores, k, tol, what=""):
    """gpu_ids: the GPU's k ids.  oracle_scores: fp64 score of EVERY eligible id (array indexed by id, or dict).
    Accepts any set that differs from the oracle's only by elements within tol of the k-th score."""
    gpu_ids = [int(i) for i in gpu_ids]
    assert len(set(gpu_ids)) == len(gpu_ids), f"{what}: duplicate ids"
    if isinstance(oracle_scores, dict):
        ids = np.fromiter(oracle_scores.keys(), dtype=np.int64)
        sc = np.fromiter(oracle_scores.values(), dtype=np.float64)
    else:
        sc = np.asarray(oracle_scores, dtype=np.float64)
        ids = np.arange(sc.shape[0])
    assert len(gpu_ids) == min(k, len(ids)), f"{what}: {len(gpu_ids)} ids, expected {min(k, len(ids))}"
    order = np.lexsort((ids, -sc))[:k]
    boundary = sc[order[-1]]
    lookup = dict(zip(ids.tolist(), sc.tolist()))
    oracle_set = set(ids[order].tolist())
    for i in gpu_ids:
        assert i in lookup, f"{what}: id {i} is not eligible"
        assert lookup[i] >= boundary - tol, f"{what}: id {i} score {lookup[i]} below boundary {boundary}"
    for i in oracle_set - set(gpu_ids):
        assert lookup[i] <= boundary + tol, f"{what}: oracle id {i} score {lookup[i]} missing (boundary {boundary})"
    return len(oracle_set & set(gpu_ids)) / max(1, len(oracle_set))


def assert_sorted_desc(scores, ids, what=""):
    s = np.asarray(scores)
    i = np.asarray(ids)
    assert np.all(s[:-1] >= s[1:]), f"{what}: scores not non-increasing"
    tie = s[:-1] == s[1:]
    assert np.all(i[:-1][tie] < i[1:][tie]), f"{what}: equal scores not in ascending id order"


def assert_scores_close(got, ref, logit_scale=1.0, what=""):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    fin = np.isfinite(ref)
    assert np.array_equal(np.isfinite(got), fin), f"{what}: finite pattern differs"
    err = np.abs(got[fin] - ref[fin])
    lim = RTOL * np.abs(ref[fin]) + ATOL_UNIT * logit_scale
    assert np.all(err <= lim), f"{what}: max err {err.max():.3e}, worst ratio {(err / lim).max():.2f}"
    return float(err.max()) if err.size else 0.0
