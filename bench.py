#!/usr/bin/env python3
"""Benchmark of the two-stage retrieval hot path (h-indexer + MoL top-k) on one MI355X.

One "step" = one query batch through the whole path: hindexer_topk (sample, threshold, corpus scan + filter,
select K') followed by mol_topk (gather, component logits, gating, softmax, weighted sum, top-k).  All inputs
(corpus cache, queries) are resident in HBM before the timed region.  Prints ONE JSON line.

Default workload: the 100M-item configuration (N=1e8, B=32, K'=1e5, P=8x8, d_P=64, H=128, k=100), synthetic
cluster-mixture data generated on the device.  After the timed region the same process measures, untimed: the
per-kernel breakdown, the memory-system ceilings (a bare read of the stage-1 table, a bare gather with the scoring
kernel's access pattern), the accuracy of what the timed steps returned against the CPU oracle, and the oracle's own
speed on a bounded slice of the workload.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0

# context only: the paper's serving latency for MoL + h-indexer on its (unnamed) production GPU, Section 5.3
PAPER_CONTEXT = {"median_latency_ms_incl_batching_wait": 30.0, "hardware": "unnamed production GPU", "source": "Section 5.3"}

CSRC = os.path.join(ROOT, "paper_2306_04039_amd", "csrc")
KERNEL_SOURCES = {  # the files a kernel is compiled from: their hash ties a profiler counter to the code that produced it
    "k_stage1_scan": ("stage1.hip", "common.hpp", "msel.hpp", "select.hpp"),
    "k_mol_score": ("mol.hip", "common.hpp"),
}


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def source_hash(kernel):
    h = hashlib.sha256()
    for name in KERNEL_SOURCES[kernel]:
        with open(os.path.join(CSRC, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def pmc_table():
    """Rows of profiles/pmc_table.md: hardware-counter readings from rocprofv3 --pmc runs of this script, each tied to
    the hash of the kernel's sources at the time of the run.  {(kernel, variant, source hash): {column: float}}."""
    path = os.path.join(ROOT, "profiles", "pmc_table.md")
    rows = {}
    if not os.path.exists(path):
        return rows
    header = None
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if not line.lstrip().startswith("|") or set(line.strip()) <= set("|-: "):
            continue
        if header is None:
            header = cells
            continue
        rec = dict(zip(header, cells))
        vals = {}
        for key, v in rec.items():
            try:
                vals[key] = float(v)
            except ValueError:
                pass
        rows[(rec.get("kernel"), rec.get("variant"), rec.get("source sha16"))] = vals
    return rows


def counters_for(kernel, variant):
    """The table row measured on exactly the sources that are compiled now, else None (a stale figure is not printed)."""
    return pmc_table().get((kernel, variant, source_hash(kernel)))


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


def bits(t):
    import numpy as np
    import torch
    t = t.detach().cpu().contiguous()
    return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()


def oracle_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] + [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def cpu_baseline(wl, items, q, gw, n_sub, kp_sub):
    """The oracle, as it stands, on a bounded slice of the same workload; scaled linearly to the full batch."""
    import numpy as np
    from oracle import retrieval_oracle as orc

    B = wl.B
    n_sub = min(n_sub, wl.N)
    x1 = bits(items["x1"][:n_sub])
    q1 = bits(q["q1"])
    n_mol = min(n_sub, 200_000)               # MoL candidates of the slice are drawn from the first n_mol items
    G = bits(items["G"][:n_mol])
    gx = bits(items["gx"][:n_mol])
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
    return {
        "value": B / (t_stage1_full + t_mol_full),
        "unit": "queries/s",
        "cores": oracle_threads(),
        "kind": "oracle",
        "sample": (f"all {B} queries; stage 1 (fp64 scores + full sort) on the first {n_sub} of {wl.N} items "
                   f"({t1 - t0:.1f}s, scaled x{wl.N / n_sub:.1f}); MoL + top-k on {kp_sub} of {wl.Kp} candidates per query "
                   f"({t3 - t2:.1f}s, scaled x{wl.Kp / kp_sub:.1f})"),
    }


def oracle_exact_stage1_topk(x1_store, q1_store, x1_real, q1_real, nq, Kp, margin, chunk=10_000_000):
    """The oracle's exact top-K' (fp64 scores of the stored bits, score desc / index asc) for the first nq queries.
    The corpus does not fit the host, so torch on the device only PRE-FILTERS: it keeps every item whose fp32 score is
    within `margin` of the fp32 K'-th score (fp32 accumulation errs by < 2e-6 here, so no member of the fp64 top-K' can
    be lost); the oracle then scores and sorts that superset.  x1_store / q1_store are the tensors the oracle reads
    (int8 codes for a quantised stage 1), x1_real / q1_real only rank the pre-filter (same tensors unless quantised)."""
    import numpy as np
    import torch
    from oracle import retrieval_oracle as orc
    N = x1_real.shape[0]
    qt = q1_real[:nq].float().t().contiguous()
    s32 = torch.empty(nq, N, dtype=torch.float32, device=x1_real.device)
    for lo in range(0, N, chunk):
        s32[:, lo:lo + chunk] = (x1_real[lo:lo + chunk].float() @ qt).t()
    out = []
    for b in range(nq):
        kth = torch.topk(s32[b], Kp).values[-1]
        ids = torch.nonzero(s32[b] >= kth - margin).flatten()
        s64 = orc.stage1_scores(bits(q1_store[b:b + 1]), bits(x1_store[ids]))[0]
        top_ids, _ = orc.topk_desc(s64, Kp, ids.cpu().numpy())
        out.append(set(top_ids.tolist()))
    del s32
    return out


def recall_vs(sets, cand_idx, counts, Kp):
    hit = 0
    for b, want in enumerate(sets):
        got = cand_idx[b, : int(counts[b])].cpu().numpy().tolist()
        hit += len(want.intersection(got))
    return hit / float(len(sets) * Kp)


def accuracy_report(wl, items, q, model_of, out_idx, out_score, cand_idx, nq_full):
    """Against the CPU oracle: relative error of every returned (query, item) score, and -- for the first nq_full queries,
    whose K' candidates the oracle scores in full -- how much of the oracle's top-k the returned top-k holds."""
    import numpy as np
    from oracle import retrieval_oracle as orc
    B, k = out_idx.shape
    Fb, gub = bits(q["F"]), bits(q["gu"])
    idx = out_idx.cpu().numpy()
    sc = out_score.cpu().numpy().astype(np.float64)
    rel, abs_err = [], []
    for b in range(B):
        ok = idx[b] >= 0
        rows = out_idx[b][out_idx[b] >= 0].long()
        model = model_of(rows)
        ref = orc.mol_scores_for(model, orc.as_f64(Fb[b]), orc.as_f64(gub[b]), np.arange(rows.numel()))
        err = np.abs(sc[b][ok] - ref)
        abs_err.append(err)
        big = np.abs(ref) > 0.1 * wl.logit_scale
        rel.append(err[big] / np.abs(ref[big]))
    rel = np.concatenate(rel) if rel else np.zeros(0)
    abs_err = np.concatenate(abs_err)
    agree, within = [], True
    for b in range(min(nq_full, B)):
        if cand_idx is not None:
            rows = cand_idx[b][cand_idx[b] >= 0].long()
        else:                                                    # exhaustive: every item is a candidate
            import torch
            rows = torch.arange(items["G"].shape[0], device=out_idx.device)
        ids = rows.cpu().numpy()
        phi = orc.mol_scores_for(model_of(rows), orc.as_f64(Fb[b]), orc.as_f64(gub[b]), np.arange(ids.shape[0]))
        top_ids, top_sc = orc.topk_desc(phi, k, ids)
        got = [i for i in idx[b].tolist() if i >= 0]
        agree.append(len(set(top_ids.tolist()) & set(got)) / float(len(top_ids)))
        lookup = dict(zip(ids.tolist(), phi.tolist()))
        tol = 2e-3 * abs(top_sc[-1]) + 1e-4 * wl.logit_scale
        within &= all(lookup[i] >= top_sc[-1] - tol for i in got)
    return {
        "reference": "CPU oracle (fp64) on the same stored bits",
        "pairs": int(abs_err.size),
        "score_max_rel_err": float(rel.max()) if rel.size else None,
        "score_p99_rel_err": float(np.quantile(rel, 0.99)) if rel.size else None,
        "score_max_abs_err": float(abs_err.max()) if abs_err.size else None,
        "tolerance": "2e-3 relative + 1e-4 * logit_scale",
        "topk_agreement": float(np.mean(agree)) if agree else None,
        "topk_agreement_queries": len(agree),
        "topk_differences_within_tolerance": bool(within) if agree else None,
    }


def time_launches(fn, reps):
    import torch
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def measured_ceilings(m, corpus, x1, cand_idx, dev, gather_bytes):
    """What the memory system delivers to kernels that only move the bytes (best of a few launch shapes)."""
    import torch
    sink = torch.zeros(64, dtype=torch.int32, device=dev)
    out = {}
    if x1 is not None:
        nbytes = x1.numel() * x1.element_size()
        best = min((time_launches(lambda: m.bench_stream_read(x1, blocks, sink), 5), blocks)
                   for blocks in (2048, 4096, 8192, 16384, 32768))
        out["stream_read"] = {"bytes": nbytes, "ms": best[0], "GBps": nbytes / (best[0] * 1e-3) / 1e9,
                              "frac_of_hbm_peak": nbytes / (best[0] * 1e-3) / 1e9 / HBM_PEAK_GBS, "blocks": best[1]}
    if cand_idx is not None:
        best = min((time_launches(lambda: m.bench_gather(corpus, cand_idx, blocks, sink), 5), blocks)
                   for blocks in (512, 1024, 2048, 4096, 8192, 16384))
        out["gather"] = {"bytes": gather_bytes, "ms": best[0], "GBps": gather_bytes / (best[0] * 1e-3) / 1e9,
                         "frac_of_hbm_peak": gather_bytes / (best[0] * 1e-3) / 1e9 / HBM_PEAK_GBS, "blocks": best[1]}
    return out


def exhaustive(args, m, wl, dev):
    """The exhaustive configuration: MoL over every item for every query, then the top-k (no stage 1).  The scoring kernel
    is a dense contraction on the matrix cores with a vector epilogue; the line reports the model arithmetic against the
    bf16 MFMA peak."""
    import numpy as np
    import torch
    from oracle import retrieval_oracle as orc
    items, q, gw = generate(wl, dev)
    corpus = m.mol_corpus_pack(None, items["G"], items["gx"], gw.W1, gw.b1, gw.W2, gw.b2, k_u=wl.k_u,
                               logit_scale=wl.logit_scale, act=wl.act, borrow=True)
    B, k = wl.B, wl.k
    ws = torch.empty(m.mol_workspace_bytes(corpus, B, 0, k), dtype=torch.uint8, device=dev)
    out = (torch.empty(B, k, dtype=torch.int32, device=dev), torch.empty(B, k, dtype=torch.float32, device=dev))
    steps, warmup = args.steps, args.warmup
    for _ in range(warmup):
        m.mol_topk(corpus, q["F"], q["gu"], None, k, workspace=ws, out=out)
    torch.cuda.synchronize()
    m.profile_read()
    m.profile_enable(True, slots=["mol_score"])
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        m.mol_topk(corpus, q["F"], q["gu"], None, k, workspace=ws, out=out)
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    m.profile_enable(False)
    mol_ms, mol_n = m.profile_read()["mol_score"]
    lat = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    m.profile_enable(True)
    m.mol_topk(corpus, q["F"], q["gu"], None, k, workspace=ws, out=out)
    torch.cuda.synchronize()
    m.profile_enable(False)
    prof = m.profile_read()
    ms_per_step = wall * 1e3 / steps
    flops = B * wl.N * (2 * wl.P * wl.d_p + 4 * wl.P * wl.H)
    launch_ms = mol_ms / max(1, mol_n)
    achieved = flops / (launch_ms * 1e-3) / 1e12
    ctr = counters_for("k_mol_score", wl.name)
    result = {
        "metric": "queries/s + p50 batch latency, exhaustive MoL top-100 over 1M items (no h-indexer), 1 GPU",
        "value": B / (ms_per_step * 1e-3), "unit": "queries/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "p50_batch_latency_ms": lat[len(lat) // 2], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: N={wl.N}, B={B}, exhaustive (cand_idx = NULL), P={wl.k_u}x{wl.k_x}, d_P={wl.d_p}, H={wl.H}, k={k}"},
        "roofline": {"kernel": "k_mol_score (item-stationary exhaustive form)", "bound": "mfma", "achieved": achieved,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                     "algorithmic_flops": flops, "avg_launch_ms": launch_ms, "launches": mol_n,
                     "note": "model arithmetic 2*P*d_P + 4*P*H flop per (query, item) pair; the kernel also runs a vector "
                             "epilogue per pair (activation, operand conversion, softmax)",
                     "mfma_busy_frac_rocprof": ctr.get("MFMA busy frac") if ctr else None,
                     "valu_busy_frac_rocprof": ctr.get("VALU busy frac") if ctr else None},
        "kernels_ms_per_step": {name: v[0] for name, v in prof.items() if v[1]},
        "paper_context": PAPER_CONTEXT,
    }

    def model_of(rows):
        return orc.MolModel(bits(items["G"][rows]), bits(items["gx"][rows]), bits(gw.W1), bits(gw.b1), bits(gw.W2),
                            bits(gw.b2), wl.logit_scale, wl.act)

    if not args.no_accuracy:
        log("comparing the returned results with the CPU oracle ...")
        result["accuracy"] = accuracy_report(wl, items, q, model_of, out[0], out[1], None, 2)
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a slice of the workload ...")
        nq, n_sub = min(B, 8), min(wl.N, 100_000)
        model = orc.MolModel(bits(items["G"][:n_sub]), bits(items["gx"][:n_sub]), bits(gw.W1), bits(gw.b1), bits(gw.W2),
                             bits(gw.b2), wl.logit_scale, wl.act)
        t0 = time.perf_counter()
        orc.mol_topk(model, bits(q["F"][:nq]), bits(q["gu"][:nq]), None, k)
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": nq / (dt * wl.N / n_sub), "unit": "queries/s", "cores": oracle_threads(),
                                  "kind": "oracle",
                                  "sample": f"{nq} of {B} queries over the first {n_sub} of {wl.N} items ({dt:.1f}s, scaled x{wl.N / n_sub:.1f} in items)"}
    print(json.dumps(result), flush=True)


def cold_cache_ms(args, m, wl, items, q, gw, q1, x1, steps):
    """Small corpora sit in the 256 MB last-level cache between steps.  This variant rotates over enough separately
    packed copies of the corpus (at least 3, at least 1 GiB together) that every step finds its tables in HBM."""
    import torch
    per_copy = sum(items[key].numel() * items[key].element_size() for key in ("x1", "G", "gx"))
    copies = max(3, -(-(1 << 30) // per_copy))
    corpora = []
    for _ in range(copies):
        c_items = {key: items[key].clone() for key in ("G", "gx")}
        c_x1 = x1.clone()
        corpora.append((m.mol_corpus_pack(c_x1, c_items["G"], c_items["gx"], gw.W1, gw.b1, gw.W2, gw.b2, k_u=wl.k_u,
                                          logit_scale=wl.logit_scale, act=wl.act, borrow=True), c_x1, c_items))
    B, Kp, k = wl.B, wl.Kp, wl.k
    dev = x1.device
    lam = m.hindexer_default_lambda(corpora[0][0], Kp)
    ws1 = torch.empty(m.hindexer_workspace_bytes(corpora[0][0], B, Kp, lam), dtype=torch.uint8, device=dev)
    ws2 = torch.empty(m.mol_workspace_bytes(corpora[0][0], B, Kp, k), dtype=torch.uint8, device=dev)
    out1 = (torch.empty(B, Kp, dtype=torch.int32, device=dev), torch.empty(B, Kp, dtype=torch.float32, device=dev),
            torch.empty(B, dtype=torch.int32, device=dev))
    out2 = (torch.empty(B, k, dtype=torch.int32, device=dev), torch.empty(B, k, dtype=torch.float32, device=dev))

    def step(i):
        c = corpora[i % copies][0]
        m.hindexer_topk(c, q1, Kp, lam=lam, seed=1000 + i, mode=args.mode, workspace=ws1, out=out1)
        m.mol_topk(c, q["F"], q["gu"], out1[0], k, workspace=ws2, out=out2, cand_count=out1[2])

    for i in range(copies):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    for c, _, _ in corpora:
        c.free()
    return {"ms_per_step": ms, "queries_per_s": B / (ms * 1e-3), "corpus_copies": copies,
            "bytes_per_copy": per_copy, "note": "rotating over separately packed copies of the corpus so that no step finds its tables in the last-level cache"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C4", choices=["C1", "C2", "C3", "C4", "C5"],
                    help="C4 is the workload the metric is quoted on; C5 is the exhaustive-MoL configuration (no stage 1)")
    ap.add_argument("--n-items", type=int, default=0, help="override N (debugging; the result is then not the named workload)")
    ap.add_argument("--no-deferred", action="store_true", help="skip the run with MOL_HINDEXER_DEFER_REDO")
    ap.add_argument("--mode", type=int, default=0, help="0 = exact-on-success h-indexer (default), 1 = Algorithm 2 as written")
    ap.add_argument("--stage1", default="config", choices=["config", "int8"],
                    help="int8: quantise the stage-1 table and queries (Section 4.1.1) and run the h-indexer on INT8 operands; "
                         "a different arithmetic from the named workload, reported as such")
    ap.add_argument("--gate", default="config", choices=["config", "decomposed"],
                    help="decomposed: Algorithm 1's gate (user / item / cross MLPs, uw*xw + cw, SiLU) instead of the workload's "
                         "concatenated MLP; a different model, reported as such")
    ap.add_argument("--gen-items", action="store_true",
                    help="generate the last 2 of the k_x item-side embeddings on the fly from a cached 32-d seed (Section 3.1) instead "
                         "of caching them; a different model (fewer bytes gathered per candidate, more matrix-core work), reported as such")
    ap.add_argument("--lam", type=int, default=0, help="h-indexer sample size (default: the library's, max(1 %% of N, 256 N / K'))")
    ap.add_argument("--in-flight", type=int, default=2,
                    help="after the timed region, also run the steps with this many batches in flight on separate streams and report "
                         "that throughput beside the headline (1 = skip)")
    ap.add_argument("--graph", action="store_true",
                    help="also record the step into a HIP graph and time its replays (no faster than eager launches on this "
                         "runtime: the time between dependent kernels is the device's, not the host's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-accuracy", action="store_true", help="skip the comparison of the returned results with the CPU oracle")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the bare read / bare gather ceiling measurements")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region, run a plain 1 GiB device copy three times (gives profilers' byte counters a kernel of known traffic)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the retrieval path on ONE GPU only (the paper's inference path is single-GPU); "
              "--gpus N with N > 1 is not supported.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2306_04039_amd as m

    m.load_library()                      # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = build_workload(args.workload, args.n_items)
    log(f"workload {wl.name}: N={wl.N} B={wl.B} K'={wl.Kp} P={wl.k_u}x{wl.k_x} d_P={wl.d_p} H={wl.H} k={wl.k}")

    if wl.Kp == 0:
        return exhaustive(args, m, wl, dev)
    gen = None
    if args.gen_items:
        import synth
        K_G, D_S, D_HG = 2, 32, 64
        items, _, _ = generate(wl.replace(k_x=wl.k_x - K_G), dev)       # the cache holds k_x - 2 embeddings per item
        cen = synth.make_centres(wl, dev)
        q, gw = synth.make_queries(wl, cen), synth.make_gate_weights(wl, dev)
        gen = {"k_g": K_G, "d_s": D_S, "seed": synth.make_item_seeds(wl, cen, D_S), "mlp": synth.make_gen_mlp(wl, dev, K_G, D_S, D_HG)}
    else:
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
                                   logit_scale=wl.logit_scale, act=wl.act, borrow=True,
                                   item_seed=gen["seed"] if gen else None, gen_mlp=gen["mlp"] if gen else None)
    log(f"mol_corpus_pack: {time.time() - t0:.1f}s")

    B, Kp, k = wl.B, wl.Kp, wl.k
    lam = args.lam if args.lam > 0 else m.hindexer_default_lambda(corpus, Kp)
    ws1 = torch.empty(m.hindexer_workspace_bytes(corpus, B, Kp, lam), dtype=torch.uint8, device=dev)
    ws2 = torch.empty(m.mol_workspace_bytes(corpus, B, Kp, k), dtype=torch.uint8, device=dev)
    out1 = (torch.empty(B, Kp, dtype=torch.int32, device=dev), torch.empty(B, Kp, dtype=torch.float32, device=dev),
            torch.empty(B, dtype=torch.int32, device=dev))
    out2 = (torch.empty(B, k, dtype=torch.int32, device=dev), torch.empty(B, k, dtype=torch.float32, device=dev))

    def step(i, mode=args.mode):
        m.hindexer_topk(corpus, q1, Kp, lam=lam, seed=1000 + i, mode=mode, workspace=ws1, out=out1)
        m.mol_topk(corpus, q["F"], q["gu"], out1[0], k, workspace=ws2, out=out2, cand_count=out1[2])

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
    final_idx, final_score, final_cand = out2[0].clone(), out2[1].clone(), out1[0].clone()

    # the same steps with the exact redo left to the caller (MOL_HINDEXER_DEFER_REDO): the nine launches of the redo return
    # at once when no query needs them but still take their place in the stream.  Reported beside the headline, which
    # keeps the redo on the device; valid only while every query completes (checked), the usual case.
    deferred = None
    if not args.no_deferred:
        dmode = args.mode | m.HINDEXER_DEFER_REDO
        for i in range(args.warmup):
            step(i, dmode)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(args.warmup + i, dmode)
        torch.cuda.synchronize()
        d_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        deferred = {"ms_per_step": d_ms, "queries_per_s": B / (d_ms * 1e-3),
                    "every_query_completed": bool(int(out1[2].min()) >= 0),
                    "outputs_identical_to_the_default_run": bool(torch.equal(out2[0], final_idx) and torch.equal(out2[1], final_score)),
                    "note": "hindexer_topk with MOL_HINDEXER_DEFER_REDO: a query the sample misleads comes back flagged for the caller to resubmit instead of being redone on the device"}

    # the same steps with two batches in flight (two streams, each with its own workspaces and outputs): the small,
    # latency-bound kernels of one batch run beside the bandwidth-bound ones of the other.  Reported beside the headline,
    # which stays one batch at a time.
    pipelined = None
    if args.in_flight > 1:
        slots = []
        for _ in range(args.in_flight):
            slots.append((torch.cuda.Stream(),
                          torch.empty_like(ws1), torch.empty_like(ws2),
                          tuple(torch.empty_like(t) for t in out1), tuple(torch.empty_like(t) for t in out2)))

        def pstep(i):
            st, w1, w2, o1, o2 = slots[i % args.in_flight]
            with torch.cuda.stream(st):
                m.hindexer_topk(corpus, q1, Kp, lam=lam, seed=1000 + i, mode=args.mode, workspace=w1, out=o1)
                m.mol_topk(corpus, q["F"], q["gu"], o1[0], k, workspace=w2, out=o2, cand_count=o1[2])

        torch.cuda.synchronize()
        for i in range(2 * args.in_flight):
            pstep(i)
        torch.cuda.synchronize()
        n_p = args.steps * args.in_flight
        t0 = time.perf_counter()
        for i in range(n_p):
            pstep(args.warmup + i)
        torch.cuda.synchronize()
        p_ms = (time.perf_counter() - t0) * 1e3 / n_p
        same = bool(all(torch.equal(sl[4][0], final_idx) and torch.equal(sl[4][1], final_score) for sl in slots))
        pipelined = {"in_flight": args.in_flight, "steps": n_p, "ms_per_step": p_ms, "queries_per_s": B / (p_ms * 1e-3),
                     "outputs_identical_to_the_single_stream_run": same,
                     "note": "batches alternate between streams; every stream has its own workspaces and outputs"}
        del slots

    # the same step recorded once into a HIP graph (both calls launch kernels only) and replayed: what a serving loop
    # with fixed buffers would do.  Reported beside the headline, which stays eager launches; the sample seed is a
    # kernel argument, so every replay draws the same sample (the results do not depend on it in this mode).
    graph_replay = None
    if args.graph:
        gstream = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=gstream):
            step(0)
        torch.cuda.synchronize()
        for _ in range(max(2, args.warmup)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        graph_replay = {"steps": args.steps, "ms_per_step": g_ms, "queries_per_s": B / (g_ms * 1e-3),
                        "outputs_identical_to_the_eager_run": bool(torch.equal(out2[0], final_idx) and torch.equal(out2[1], final_score)),
                        "note": "one captured step (hindexer_topk -> mol_topk, kernel nodes only) replayed back to back"}
        del graph

    scan_ms, scan_n = prof_scan["scan_filter"]
    scan_bytes = wl.N * wl.d1 * (1 if int8 else (4 if wl.stage1_dtype == "f32" else 2))
    achieved = scan_bytes / (scan_ms / scan_n * 1e-3) / 1e9 if scan_n else 0.0
    mol_ms, mol_n = prof["mol_score"]
    k_cached = wl.k_x - (gen["k_g"] if gen else 0)
    bytes_per_cand = k_cached * wl.d_p * 2 + (gen["d_s"] * 2 if gen else 0) + (wl.P * 4 if decomposed else wl.H * 2) + 4 + 4
    gather_bytes = B * Kp * bytes_per_cand
    mol_flops = B * Kp * (2 * wl.P * wl.d_p + 4 * wl.P * wl.H)

    # hardware-counter readings: only those taken on exactly the sources compiled now (profiles/pmc_table.md)
    variant = wl.name + ("/int8" if int8 else "")
    scan_ctr = counters_for("k_stage1_scan", variant) if (not args.n_items and args.mode == 0) else None
    mol_ctr = counters_for("k_mol_score", wl.name) if (not args.n_items and not decomposed and not gen) else None
    traffic = None
    if scan_ctr and "FETCH_SIZE KiB" in scan_ctr:
        traffic = (scan_ctr["FETCH_SIZE KiB"] * scan_ctr.get("fetch scale", 1.0)
                   + scan_ctr.get("WRITE_SIZE KiB", 0.0) * scan_ctr.get("write scale", 1.0)) * 1024.0

    headline = wl.name.startswith("C4")
    result = {
        "metric": ("queries/s + p50 batch latency, 100M-item h-indexer+MoL top-100, 1 GPU" if headline else
                   f"queries/s + p50 batch latency, h-indexer+MoL top-{k}, 1 GPU (workload {wl.name})"),
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
                               f"h-indexer mode {args.mode}, lambda={lam}" + (", INT8 stage 1" if int8 else "") + (", decomposed gate (Algorithm 1)" if decomposed else "")
                               + (f", {gen['k_g']} of {wl.k_x} item-side embeddings generated on the fly from a {gen['d_s']}-d seed (Section 3.1)" if gen else "")},
        "roofline": {"kernel": "k_stage1_scan (corpus scan + threshold filter)", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_unit": "bytes per launch (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, calibrated; null unless measured on the sources compiled now)",
                     "algorithmic_bytes": scan_bytes,
                     "avg_launch_ms": scan_ms / max(1, scan_n), "launches": scan_n},
        "kernels_ms_per_step": {name: v[0] / args.steps for name, v in prof.items() if v[1]},
        "kernels_note": "from a second, untimed set of steps with every kernel group bracketed by events",
        "mol_stage": {"bytes_gathered_per_candidate": bytes_per_cand, "gather_GBps": gather_bytes / (mol_ms / max(1, mol_n) * 1e-3) / 1e9 if mol_n else 0.0,
                      "gather_frac_of_hbm_peak": (gather_bytes / (mol_ms / max(1, mol_n) * 1e-3) / 1e9 / HBM_PEAK_GBS) if mol_n else 0.0,
                      "model_TFLOPs": mol_flops / (mol_ms / max(1, mol_n) * 1e-3) / 1e12 if mol_n else 0.0,
                      "model_frac_of_bf16_mfma_peak": (mol_flops / (mol_ms / max(1, mol_n) * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS) if mol_n else 0.0,
                      "mfma_busy_frac_rocprof": mol_ctr.get("MFMA busy frac") if mol_ctr else None},
        "paper_context": PAPER_CONTEXT,
    }
    if deferred:
        result["deferred_redo"] = deferred
    if pipelined:
        result["pipelined"] = pipelined
    if graph_replay:
        result["graph_replay"] = graph_replay

    if not args.no_ceiling and not decomposed:
        ceil = measured_ceilings(m, corpus, x1, None if gen else final_cand, dev, gather_bytes)
        result["measured_ceiling"] = ceil
        if "stream_read" in ceil and scan_n:
            result["roofline"]["frac_of_measured_stream_read"] = ceil["stream_read"]["ms"] / (scan_ms / scan_n)
        if "gather" in ceil and mol_n:
            result["mol_stage"]["frac_of_measured_gather"] = ceil["gather"]["ms"] / (mol_ms / mol_n)

    if not args.no_accuracy and not decomposed:
        from oracle import retrieval_oracle as orc
        log("comparing the returned results with the CPU oracle ...")

        def model_of(rows):
            extra = dict(seed=bits(gen["seed"][rows]), gen_mlp=tuple(bits(t) for t in gen["mlp"])) if gen else {}
            return orc.MolModel(bits(items["G"][rows]), bits(items["gx"][rows]), bits(gw.W1), bits(gw.b1), bits(gw.W2),
                                bits(gw.b2), wl.logit_scale, wl.act, **extra)

        nq = min(4, B)
        result["accuracy"] = accuracy_report(wl, items, q, model_of, final_idx, final_score, final_cand, nq)
        # stage-1 recall@K' against the oracle's exact top-K' of the table the h-indexer scanned, both modes
        exact_sets = oracle_exact_stage1_topk(x1, q1, x1, q1, nq, Kp, 1.0 if int8 else 1e-4)
        rec = {}
        for mode, name in ((0, "exact_on_success"), (1, "algorithm2_as_written")):
            m.hindexer_topk(corpus, q1, Kp, lam=lam, seed=1000, mode=mode, workspace=ws1, out=out1)
            torch.cuda.synchronize()
            rec[name] = recall_vs(exact_sets, out1[0], out1[2].cpu().numpy(), Kp)
        rec["queries"] = nq
        rec["reference"] = "oracle exact top-K' (fp64 scores, full sort) of the scanned table"
        result["stage1_recall_at_Kp"] = rec
        if int8:   # how much of the unquantised table's exact top-K' the quantised stage 1 keeps (a property of the scheme)
            real_sets = oracle_exact_stage1_topk(items["x1"], q["q1"], items["x1"], q["q1"], nq, Kp, 1e-4)
            m.hindexer_topk(corpus, q1, Kp, lam=lam, seed=1000, mode=0, workspace=ws1, out=out1)
            torch.cuda.synchronize()
            result["int8_stage1_recall_vs_unquantised_topKp"] = recall_vs(real_sets, out1[0], out1[2].cpu().numpy(), Kp)

    if wl.N <= 1_000_000 and not decomposed and not gen and not args.no_ceiling:
        result["cold_cache"] = cold_cache_ms(args, m, wl, items, q, gw, q1, x1, args.steps)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline and not decomposed and not gen:
        log("timing the CPU oracle on a slice of the workload ...")
        result["cpu_baseline"] = cpu_baseline(wl, items, q, gw, min(wl.N, 4_000_000), 16384)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
