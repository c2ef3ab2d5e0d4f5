#!/usr/bin/env python3
"""Benchmark of the two-stage retrieval hot path (h-indexer + MoL top-k) on one MI355X.

One "step" = one query batch through the whole path: hindexer_topk (sample, threshold, corpus scan + filter,
select K') followed by mol_topk (gather, component logits, gating, softmax, weighted sum, top-k).  All inputs
(corpus cache, queries) are resident in HBM before the timed region.  Prints ONE JSON line.

Default workload: the 100M-item configuration (N=1e8, B=32, K'=1e5, P=8x8, d_P=64, H=128, k=100), synthetic
cluster-mixture data generated on the device.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes one launch of the corpus scan moves on the default workload, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this script (KiB per dispatch), each scaled by what the same counter reads for a 1 GiB device copy (--calibrate-copy):
# FETCH_SIZE counts half the bytes (x2.000), WRITE_SIZE all of them (x1.000).  Re-measure when the scan kernel changes.
# matrix-core busy fraction of the MoL kernel from a rocprofv3 --pmc run of this script (profiles/k_mol_score_C4-100M.md)
MOL_MFMA_BUSY_FRAC = {"C4-100M": 0.157}
SCAN_TRAFFIC_KIB = {("C4-100M", False): {"fetch": 6250157.8, "fetch_scale": 2.0, "write": 31848.2, "write_scale": 1.0},
                    ("C4-100M", True): {"fetch": 3125108.3, "fetch_scale": 2.0, "write": 33815.5, "write_scale": 1.0}}  # key: (workload, int8 stage 1)

# context only: the paper's serving latency for MoL + h-indexer on its (unnamed) production GPU, Section 5.3
PAPER_CONTEXT = {"median_latency_ms_incl_batching_wait": 30.0, "hardware": "unnamed production GPU", "source": "Section 5.3"}


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def build_workload(name, n_override):
    import synth
    wl = synth.CONFIGS[name]
    if n_override:
        wl = wl.replace(N=n_override, Kp=min(wl.Kp, max(1, n_override // 8)))
    return wl


def generate(wl, dev):
    import torch
    import synth
    cen = synth.make_centres(wl, dev)
    t0 = time.time()

    def progress(i, n):
        if i % 10 == 0 or i == n:
            log(f"generated {i}/{n} item chunks ({time.time() - t0:.0f}s)")

    items = synth.make_items(wl, cen, progress=progress)
    q = synth.make_queries(wl, cen)
    gw = synth.make_gate_weights(wl, dev)
    torch.cuda.synchronize()
    return items, q, gw


def cpu_baseline(wl, items, q, gw, n_sub, kp_sub):
    """The oracle, as it stands, on a bounded slice of the same workload; scaled linearly to the full batch."""
    import numpy as np
    import torch
    from oracle import retrieval_oracle as orc

    def bits(t):
        t = t.detach().cpu().contiguous()
        return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()

    B = wl.B
    n_sub = min(n_sub, wl.N)
    x1 = bits(items["x1"][:n_sub])
    q1 = bits(q["q1"])
    n_mol = min(n_sub, 200_000)               # MoL candidates of the slice are drawn from the first n_mol items
    G = bits(items["G"][:n_mol])
    gx = bits(items["gx_sub"][:n_mol])
    kp_sub = min(kp_sub, wl.Kp, n_mol)
    kp_stage1 = max(1, int(round(wl.Kp * n_sub / wl.N)))
    t0 = time.perf_counter()
    stage1 = orc.exact_topk_stage1(q1, x1, kp_stage1)            # fp64 scores of the slice + full sort per query
    t1 = time.perf_counter()
    model = orc.MolModel(G, gx, bits(gw.W1), bits(gw.b1), bits(gw.W2), bits(gw.b2), wl.logit_scale, wl.act)
    rng = np.random.default_rng(0)
    cand = rng.integers(0, n_mol, size=(B, kp_sub))
    t2 = time.perf_counter()
    orc.mol_topk(model, bits(q["F"]), bits(q["gu"]), cand, wl.k)
    t3 = time.perf_counter()
    del stage1
    t_stage1_full = (t1 - t0) * (wl.N / n_sub)
    t_mol_full = (t3 - t2) * (wl.Kp / kp_sub)
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    return {
        "value": B / (t_stage1_full + t_mol_full),
        "unit": "queries/s",
        "cores": int(threads),
        "kind": "oracle",
        "sample": (f"all {B} queries; stage 1 (fp64 scores + full sort) on the first {n_sub} of {wl.N} items "
                   f"({t1 - t0:.1f}s, scaled x{wl.N / n_sub:.1f}); MoL + top-k on {kp_sub} of {wl.Kp} candidates per query "
                   f"({t3 - t2:.1f}s, scaled x{wl.Kp / kp_sub:.1f})"),
    }


def stage1_recall(x1, q1, cand_idx, Kp, n_queries=4, chunk=10_000_000):
    """Share of the unquantised stage-1 top-K' (torch matmul on the stored table, first n_queries queries) that the
    candidate lists contain.  Evaluation of the quantisation only; not part of the timed path."""
    import torch
    nq = min(n_queries, q1.shape[0])
    qt = q1[:nq].float().t().contiguous()
    scores = torch.empty(nq, x1.shape[0], dtype=torch.float32, device=x1.device)
    for lo in range(0, x1.shape[0], chunk):
        scores[:, lo:lo + chunk] = (x1[lo:lo + chunk].float() @ qt).t()
    hit = 0
    for b in range(nq):
        top = torch.topk(scores[b], Kp).indices
        mark = torch.zeros(x1.shape[0], dtype=torch.bool, device=x1.device)
        mark[top] = True
        c = cand_idx[b]
        hit += int(mark[c[c >= 0].long()].sum())
    return hit / float(nq * Kp)


def exhaustive(args, m, wl, dev):
    """The exhaustive configuration: MoL over every item for every query, then the top-k (no stage 1).  The scoring kernel
    is a dense contraction (matrix cores) co-limited by its vector epilogue; the line reports the model arithmetic against
    the bf16 MFMA peak."""
    import torch
    items, q, gw = generate(wl, dev)
    corpus = m.mol_corpus_pack(None, items["G"], items["gx"], gw.W1, gw.b1, gw.W2, gw.b2, k_u=wl.k_u,
                               logit_scale=wl.logit_scale, act=wl.act, borrow=True)
    B, k = wl.B, wl.k
    ws = torch.empty(m.mol_workspace_bytes(corpus, B, 0, k), dtype=torch.uint8, device=dev)
    out = (torch.empty(B, k, dtype=torch.int32, device=dev), torch.empty(B, k, dtype=torch.float32, device=dev))
    steps, warmup = min(args.steps, 10), min(args.warmup, 2)
    for _ in range(warmup):
        m.mol_topk(corpus, q["F"], q["gu"], None, k, workspace=ws, out=out)
    torch.cuda.synchronize()
    m.profile_read()
    m.profile_enable(True, slots=["mol_score"])
    t0 = time.perf_counter()
    for _ in range(steps):
        m.mol_topk(corpus, q["F"], q["gu"], None, k, workspace=ws, out=out)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    m.profile_enable(False)
    mol_ms, mol_n = m.profile_read()["mol_score"]
    ms_per_step = wall * 1e3 / steps
    flops = B * wl.N * (2 * wl.P * wl.d_p + 4 * wl.P * wl.H)
    achieved = flops / (mol_ms / max(1, mol_n) * 1e-3) / 1e12
    print(json.dumps({
        "metric": "queries/s, exhaustive MoL top-100 over 1M items, 1 GPU", "value": B / (ms_per_step * 1e-3), "unit": "queries/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: N={wl.N}, B={B}, exhaustive, P={wl.k_u}x{wl.k_x}, d_P={wl.d_p}, H={wl.H}, k={k}"},
        "roofline": {"kernel": "k_mol_score (item-stationary exhaustive form)", "bound": "mfma", "achieved": achieved, "peak": 2500.0,
                     "unit": "TFLOP/s", "frac": achieved / 2500.0, "traffic": None, "avg_launch_ms": mol_ms / max(1, mol_n),
                     "launches": mol_n,
                     "note": "model arithmetic 2*P*d_P + 4*P*H flop per pair; the kernel is co-limited by its vector epilogue "
                             "(activation, hi/lo split, softmax: about 1000 lane-operations per pair)"},
    }), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C4", choices=["C1", "C2", "C3", "C4", "C5"],
                    help="C4 is the workload the metric is quoted on; C5 is the exhaustive-MoL configuration (no stage 1)")
    ap.add_argument("--n-items", type=int, default=0, help="override N (debugging; the result is then not the named workload)")
    ap.add_argument("--mode", type=int, default=0, help="0 = exact-on-success h-indexer (default), 1 = Algorithm 2 as written")
    ap.add_argument("--stage1", default="config", choices=["config", "int8"],
                    help="int8: quantise the stage-1 table and queries (Section 4.1.1) and run the h-indexer on INT8 operands; "
                         "a different arithmetic from the named workload, reported as such")
    ap.add_argument("--gate", default="config", choices=["config", "decomposed"],
                    help="decomposed: Algorithm 1's gate (user / item / cross MLPs, uw*xw + cw, SiLU) instead of the workload's "
                         "concatenated MLP; a different model, reported as such")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region, run a plain 1 GiB device copy three times (gives profilers' byte counters a kernel of known traffic)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the retrieval path on ONE GPU only (the paper's inference path is single-GPU); "
              "--gpus N with N > 1 is not supported.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2306_04039_amd as m

    m.load_library()                      # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = build_workload(args.workload, args.n_items)
    log(f"workload {wl.name}: N={wl.N} B={wl.B} K'={wl.Kp} P={wl.k_u}x{wl.k_x} d_P={wl.d_p} H={wl.H} k={wl.k}")

    if wl.Kp == 0:
        return exhaustive(args, m, wl, dev)
    items, q, gw = generate(wl, dev)
    t0 = time.time()
    int8 = args.stage1 == "int8"
    x1, q1 = items["x1"], q["q1"]
    if int8:
        x1 = m.quantize_int8(items["x1"], 127.0 / float(items["x1"].float().abs().max()))
        q1 = m.quantize_int8(q["q1"], 127.0 / float(q["q1"].float().abs().max()))
    decomposed = args.gate == "decomposed"
    if decomposed:
        import synth
        user_mlp, item_mlp, cross_mlp = synth.make_decomposed_gate_weights(wl, dev)
        corpus = m.mol_corpus_pack(x1, items["G"], items["gx"], *cross_mlp, k_u=wl.k_u, logit_scale=wl.logit_scale,
                                   act=wl.act, borrow=True, user_mlp=user_mlp, item_mlp=item_mlp)
    else:
        corpus = m.mol_corpus_pack(x1, items["G"], items["gx"], gw.W1, gw.b1, gw.W2, gw.b2, k_u=wl.k_u,
                                   logit_scale=wl.logit_scale, act=wl.act, borrow=True)
    log(f"mol_corpus_pack: {time.time() - t0:.1f}s")
    n_sub = min(wl.N, 4_000_000)
    items["gx_sub"] = items["gx"][:n_sub].clone()
    del items["gx"]                       # the raw item gate features are not needed after pack
    torch.cuda.empty_cache()

    B, Kp, k = wl.B, wl.Kp, wl.k
    lam = m.hindexer_default_lambda(corpus, Kp)
    ws1 = torch.empty(m.hindexer_workspace_bytes(corpus, B, Kp, lam), dtype=torch.uint8, device=dev)
    ws2 = torch.empty(m.mol_workspace_bytes(corpus, B, Kp, k), dtype=torch.uint8, device=dev)
    out1 = (torch.empty(B, Kp, dtype=torch.int32, device=dev), torch.empty(B, Kp, dtype=torch.float32, device=dev),
            torch.empty(B, dtype=torch.int32, device=dev))
    out2 = (torch.empty(B, k, dtype=torch.int32, device=dev), torch.empty(B, k, dtype=torch.float32, device=dev))

    def step(i):
        m.hindexer_topk(corpus, q1, Kp, lam=lam, seed=1000 + i, mode=args.mode, workspace=ws1, out=out1)
        m.mol_topk(corpus, q["F"], q["gu"], out1[0], k, workspace=ws2, out=out2)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # timed region: only the dominant kernel (the corpus scan) is bracketed by HIP events inside the library (each
    # bracket idles the device for about 10 us); the per-kernel breakdown comes from a second, untimed set of steps
    m.profile_read()
    m.profile_enable(True, slots=["scan_filter"])
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(args.steps):
        step(args.warmup + i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    m.profile_enable(False)
    prof_scan = m.profile_read()
    lat = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps))
    ms_per_step = wall * 1e3 / args.steps
    m.profile_enable(True)
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    m.profile_enable(False)
    prof = m.profile_read()
    counts = out1[2].cpu()
    assert int(counts.min()) >= 0, "h-indexer reported a failed query"

    scan_ms, scan_n = prof_scan["scan_filter"]
    scan_bytes = wl.N * wl.d1 * (1 if int8 else (4 if wl.stage1_dtype == "f32" else 2))
    achieved = scan_bytes / (scan_ms / scan_n * 1e-3) / 1e9 if scan_n else 0.0
    mol_ms, mol_n = prof["mol_score"]
    gather_bytes = B * Kp * (wl.k_x * wl.d_p * 2 + (wl.P * 4 if decomposed else wl.H * 2) + 4 + 4)
    mol_flops = B * Kp * (2 * wl.P * wl.d_p + 4 * wl.P * wl.H)

    traffic = None
    t = SCAN_TRAFFIC_KIB.get((wl.name, int8))
    if t and not args.n_items and args.mode == 0:
        traffic = (t["fetch"] * t["fetch_scale"] + t["write"] * t["write_scale"]) * 1024.0

    result = {
        "metric": "queries/s + p50 batch latency, 100M-item h-indexer+MoL top-100, 1 GPU",
        "value": B / (ms_per_step * 1e-3),
        "unit": "queries/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "p50_batch_latency_ms": lat[len(lat) // 2],
        "p95_batch_latency_ms": lat[min(len(lat) - 1, int(0.95 * len(lat)))],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 stage 1 (int32 scores) + bf16 MoL" if int8 else ("bf16" if wl.stage1_dtype != "f32" else "f32"),
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: N={wl.N}, B={B}, K'={Kp}, P={wl.k_u}x{wl.k_x}, d_P={wl.d_p}, H={wl.H}, k={k}, "
                               f"h-indexer mode {args.mode}, lambda={lam}" + (", INT8 stage 1" if int8 else "") + (", decomposed gate (Algorithm 1)" if decomposed else "")},
        "roofline": {"kernel": "k_stage1_scan (corpus scan + threshold filter)", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_unit": "bytes per launch (rocprofv3 --pmc, calibrated)",
                     "algorithmic_bytes": scan_bytes,
                     "avg_launch_ms": scan_ms / max(1, scan_n), "launches": scan_n},
        "kernels_ms_per_step": {name: v[0] / args.steps for name, v in prof.items() if v[1]},
        "kernels_note": "from a second, untimed set of steps with every kernel group bracketed by events",
        "mol_stage": {"gather_GBps": gather_bytes / (mol_ms / max(1, mol_n) * 1e-3) / 1e9 if mol_n else 0.0,
                      "gather_frac_of_hbm_peak": (gather_bytes / (mol_ms / max(1, mol_n) * 1e-3) / 1e9 / HBM_PEAK_GBS) if mol_n else 0.0,
                      "model_TFLOPs": mol_flops / (mol_ms / max(1, mol_n) * 1e-3) / 1e12 if mol_n else 0.0,
                      "model_frac_of_bf16_mfma_peak": (mol_flops / (mol_ms / max(1, mol_n) * 1e-3) / 1e12 / 2500.0) if mol_n else 0.0,
                      "mfma_busy_frac_rocprof": MOL_MFMA_BUSY_FRAC.get(wl.name) if not decomposed else None},
        "paper_context": PAPER_CONTEXT,
    }
    # stage-1 recall@K' against the exact top-K' of the stored (unquantised) table, first 4 queries, torch fp32 matmul
    rec = stage1_recall(items["x1"], q["q1"], out1[0], Kp)
    result["int8_stage1_recall_vs_unquantised_topKp" if int8 else "stage1_recall_at_Kp"] = rec
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline and not decomposed:
        log("timing the CPU oracle on a slice of the workload ...")
        result["cpu_baseline"] = cpu_baseline(wl, items, q, gw, n_sub, 16384)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
