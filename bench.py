#!/usr/bin/env python3
"""Benchmark of the sparse GNN hot path on one MI355X.

One "step" = one pass of the hot path over the workload with all inputs resident in HBM:
the cached-transpose lookup (a cache hit after the first call), SpMM forward Y = A X and SpMM
backward dX = A^T dY (configs 1-3), plus SDDMM where the configuration lists it, or FusedMM
forward + backward (config 4).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 0..4]

The default workload is configuration 3, the largest power-law graph (R-MAT, n = 2,449,029,
~123.6 M stored entries, d = 128), which is the one the bandwidth target is quoted on.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--shrink", type=int, default=1, help="divide the graph size (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-relabel", action="store_true",
                    help="keep the R-MAT generator's own vertex ids instead of the random relabelling (a point of "
                         "comparison, not a benchmark configuration; the workload name says so)")
    ap.add_argument("--ops", default="", help="comma-separated operations to time in place of the workload's own "
                                              "(spmm, spmm_t, sddmm, fusedmm, fusedmm_bwd); not the headline line")
    ap.add_argument("--epoch-ablation", type=int, default=0, metavar="E",
                    help="instead of the benchmark line: time E training epochs (forward + backward SpMM) with "
                         "the cached transpose and with the transpose rebuilt every epoch")
    ap.add_argument("--sweep-d", action="store_true",
                    help="instead of the benchmark line: SpMM forward time over feature widths 8..1024")
    ap.add_argument("--graph", action="store_true",
                    help="instead of the benchmark line: the step captured in a HIP graph vs launched eagerly "
                         "(matters for the launch-bound small workloads)")
    ap.add_argument("--gcn-step", action="store_true",
                    help="instead of the benchmark line: a 2-layer GCN training step (sparse ops through the "
                         "autograd wrappers, dense GEMMs through torch) with hidden width d")
    ap.add_argument("--reductions", action="store_true",
                    help="instead of the benchmark line: forward and backward time of the mean / min / max reductions")
    ap.add_argument("--flushed", action="store_true",
                    help="instead of the benchmark line: per-op time when a 1 GiB copy has swept L2 and the "
                         "Infinity Cache before every op (the small workloads otherwise run cache-warm)")
    ap.add_argument("--split-rows", type=int, default=0, metavar="T",
                    help="instead of the benchmark line: SpMM forward on the two sub-matrices made of the rows with at "
                         "most T stored entries and of the longer rows (the other rows left empty), each timed alone: "
                         "where a launch on the whole matrix spends its time")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of the benchmark line: what this box's memory system delivers to this access pattern - "
                         "a plain device copy and the library's SpMM on uniform random graphs whose dense operand has a "
                         "footprint of 2 MB ... 1.25 GB (requested gather bytes over time)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="(kept for older command lines: plain device copies of X, the known-size kernel that "
                         "scales rocprofv3 FETCH_SIZE / WRITE_SIZE readings, now always run before the timed region)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import graphgen
    import paper_2403_14853_amd as isp

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    isp.load_library()  # fails loudly when the HIP library is missing
    if args.ceilings:
        print(json.dumps(ceilings(isp)))
        return
    t0 = time.time()
    w = graphgen.make_config(args.config, shrink=args.shrink, relabel=not args.no_relabel)
    gen_s = time.time() - t0
    n, d, nnz = w.n, w.d, w.nnz
    dev = lambda a: torch.from_numpy(a).cuda()
    indptr, indices = dev(w.indptr), dev(w.indices)
    values = None if w.values is None else dev(w.values)
    X, dY = dev(w.X), dev(w.dY)
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()

    def timed(fn):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        out = fn()
        b.record(stream)
        b.synchronize()
        return out, a.elapsed_time(b)

    # the caller owns the workspaces (as at the C boundary): allocated and touched before the timed calls
    ws_a = torch.zeros(isp.csr_build_workspace(n, n, nnz), dtype=torch.uint8, device="cuda")
    A, build_ms = timed(lambda: isp.csr_build(indptr, indices, values, workspace=ws_a))
    ws_t = torch.zeros(isp.csr_transpose_workspace(A), dtype=torch.uint8, device="cuda")
    (At, _), transpose_ms = timed(lambda: isp.csr_transpose_cached(A, workspace=ws_t))
    info, info_t = A.info(), At.info()

    if args.epoch_ablation > 0:
        print(json.dumps(epoch_ablation(isp, w, indptr, indices, values, X, dY, args.epoch_ablation)))
        return
    if args.sweep_d:
        print(json.dumps(sweep_d(isp, w, A)))
        return
    if args.split_rows > 0:
        print(json.dumps(split_rows(isp, w, X, args.split_rows, max(3, args.steps // 4))))
        return
    if args.reductions:
        print(json.dumps(reductions(isp, w, A, X, dY)))
        return
    if args.gcn_step:
        print(json.dumps(gcn_step(w, indptr, indices, values, X)))
        return

    ops = list(w.ops)
    if args.config == 1:  # two-layer GCN step: forward and backward SpMM per layer
        ops = ["spmm", "spmm", "spmm_t", "spmm_t"]
    if args.ops:
        ops = args.ops.split(",")
    Y, dX = torch.empty_like(X), torch.empty_like(X)
    dA = torch.empty(nnz, dtype=torch.float32, device="cuda") if "sddmm" in ops else None
    flops_of = {"spmm": 2.0 * nnz * d, "spmm_t": 2.0 * nnz * d, "sddmm": 2.0 * nnz * d,
                "fusedmm": 4.0 * nnz * d, "fusedmm_bwd": 10.0 * nnz * d}
    run_of = {
        "spmm": lambda: isp.spmm(A, X, Y),
        "spmm_t": lambda: isp.spmm(isp.csr_transpose_cached(A)[0], dY, dX),  # cache hit every step
        "sddmm": lambda: isp.sddmm(A, dY, X, dA),
        "fusedmm": lambda: isp.fusedmm(A, X, Y),
        "fusedmm_bwd": lambda: isp.fusedmm_backward(A, X, dY, dX),
    }

    def step(events=None):
        for i, op in enumerate(ops):
            if events is not None:
                events[i][0].record(stream)
            run_of[op]()
            if events is not None:
                events[i][1].record(stream)

    for _ in range(args.warmup):
        step()
    if args.graph:
        torch.cuda.synchronize()
        eager_ms = _time_ms(step, args.steps)
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                step()
        torch.cuda.synchronize()
        g.replay()
        graph_ms = _time_ms(g.replay, args.steps)
        print(json.dumps({"what": "one step launched eagerly vs replayed from a captured HIP graph", "workload": w.name,
                          "ops": ops, "eager_ms_per_step": round(eager_ms, 4), "graph_ms_per_step": round(graph_ms, 4)}))
        return
    if args.flushed:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        warm, cold = [[] for _ in ops], [[] for _ in ops]
        for k in range(args.steps):
            for flush, acc in ((False, warm), (True, cold)):
                for i, op in enumerate(ops):
                    if flush:
                        dst.copy_(src)  # 1 GiB read + 1 GiB written: four times the Infinity Cache
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record(stream)
                    run_of[op]()
                    b.record(stream)
                    b.synchronize()
                    acc[i].append(a.elapsed_time(b))
        print(json.dumps({"what": "per-op time, back to back vs after a 1 GiB copy has flushed the caches",
                          "workload": w.name, "steps": args.steps,
                          "warm_ms": {("%d:%s" % (i, o)): round(float(np.median(warm[i])), 4) for i, o in enumerate(ops)},
                          "flushed_ms": {("%d:%s" % (i, o)): round(float(np.median(cold[i])), 4) for i, o in enumerate(ops)}}))
        return
    # plain device copy of X (reads 4 n d bytes, writes 4 n d bytes): the streaming ceiling of this machine, and the
    # known-size kernel the rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by
    for _ in range(2):
        Y.copy_(X)
    copy_ms = _time_ms(lambda: Y.copy_(X), 5 if args.copy_calibration or n * d > 1 << 20 else 50)
    copy_gbps = 2.0 * 4.0 * n * d / (copy_ms * 1e-3) / 1e9
    torch.cuda.synchronize()
    # per-op HIP events on the launch stream, recorded inside the timed region
    evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in ops]
           for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(evs[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    op_ms = [float(np.mean([evs[k][i][0].elapsed_time(evs[k][i][1]) for k in range(args.steps)]))
             for i in range(len(ops))]
    total_flops = sum(flops_of[o] for o in ops)
    value = total_flops / (ms_per_step * 1e-3) / 1e9

    # dominant kernel: the row-streaming SpMM kernel (forward launch).  Algorithmic bytes of one
    # launch = every operand moved once: CSR (8 B per row offset + 4 B index + 4 B value per
    # entry) + X read once + Y written once.
    dom = "fusedmm" if args.config == 4 else "spmm"
    if dom not in ops:  # --ops without the workload's dominant operation: report on the first one timed
        dom = ops[0]
    dom_ms = float(np.mean([op_ms[i] for i, o in enumerate(ops) if o == dom]))
    val_bytes = 4 if w.values is not None else 0
    csr_bytes = 8.0 * (n + 1) + (4.0 + val_bytes) * nnz
    alg_bytes = csr_bytes + 2.0 * 4.0 * n * d
    gather_bytes = csr_bytes + 4.0 * d * nnz + 4.0 * n * d  # every entry fetches its own X row
    achieved = alg_bytes / (dom_ms * 1e-3) / 1e9
    dom_kernel = {"fusedmm": "k_fused_grouped<g_fwd>", "spmm": "k_spmm_grouped"}.get(dom, dom)
    roofline = {
        "bound": "hbm", "kernel": dom_kernel,
        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
        "algorithmic_bytes": alg_bytes, "launch_ms": round(dom_ms, 4),
        "gather_model_bytes": gather_bytes,
        "gather_model_GBps": round(gather_bytes / (dom_ms * 1e-3) / 1e9, 1),
        # what a plain device copy of X reaches on this machine in this run (read + written bytes over time)
        "copy_ceiling_GBps": round(copy_gbps, 1),
        "achieved_frac_of_copy_ceiling": round(achieved / copy_gbps, 4),
    }
    rec = None if (args.no_relabel or args.shrink != 1 or args.ops) else counter_record(w.name, dom_kernel)
    if rec:  # counter bytes of the stored profile record over this run's launch time
        roofline["traffic"] = rec["bytes"]
        roofline["traffic_commit"] = rec["commit"]
        roofline["traffic_source"] = "profiles/counter_records.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, calibrated)"
        roofline["traffic_over_algorithmic"] = round(rec["bytes"] / alg_bytes, 2)
        roofline["traffic_GBps"] = round(rec["bytes"] / (dom_ms * 1e-3) / 1e9, 1)
        roofline["traffic_frac_of_peak"] = round(roofline["traffic_GBps"] / HBM_PEAK_GBPS, 4)
        roofline["traffic_frac_of_copy_ceiling"] = round(roofline["traffic_GBps"] / copy_gbps, 4)
        if rec["tcc_hit"] + rec["tcc_miss"] > 0:
            roofline["l2_hit_rate"] = round(rec["tcc_hit"] / (rec["tcc_hit"] + rec["tcc_miss"]), 4)

    cpu = None
    if not args.no_cpu_baseline and not args.ops:  # the oracle leg checks the workload's own dominant output
        cpu = cpu_baseline(w, Y, dom)

    out = {
        "metric": "SpMM fwd+bwd GFLOP/s (2*nnz*d/t)" if args.config != 4 else "FusedMM fwd+bwd GFLOP/s",
        "value": round(value, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "n": n, "nnz": nnz, "d": d, "ops": ops,
                   "max_degree": info["max_degree"], "hub_rows": info["n_hub_rows"],
                   "work_items": info["n_row_blocks"] + info["n_segments"]},
        "op_ms": {("%d:%s" % (i, o)): round(op_ms[i], 4) for i, o in enumerate(ops)},
        "op_gflops": {("%d:%s" % (i, o)): round(flops_of[o] / (op_ms[i] * 1e-3) / 1e9, 1) for i, o in enumerate(ops)},
        "setup_ms": {"generate_host": round(gen_s * 1e3, 1), "csr_build": round(build_ms, 3),
                     "transpose_first_call": round(transpose_ms, 3)},
        # how many backward passes the one-time transpose costs (it is cached from then on)
        "transpose_cost_in_backward_ops": round(transpose_ms / op_ms[-1], 2),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


def counter_record(workload, kernel):
    """The rocprofv3 counter readings kept for this workload's dominant kernel in profiles/counter_records.txt
    (per launch: FETCH_SIZE and WRITE_SIZE in KiB, TCC_HIT_sum, TCC_MISS_sum, the average duration of the run
    that was counted, and the commit whose kernels were measured), or None.  The calibration factors that
    turn counter KiB into bytes are lines of the same file."""
    path = os.path.join(ROOT, "profiles", "counter_records.txt")
    if not os.path.exists(path):
        return None
    factor = {"fetch_factor": 1.0, "write_factor": 1.0}
    rec = None
    for line in open(path):
        f = line.split("#")[0].split()
        if len(f) == 2 and f[0] in factor:
            factor[f[0]] = float(f[1])
        elif len(f) == 8 and f[0] == workload and f[1] == kernel:
            rec = dict(fetch_kib=float(f[2]), write_kib=float(f[3]), tcc_hit=float(f[4]), tcc_miss=float(f[5]),
                       avg_us=float(f[6]), commit=f[7])
    if rec is None:
        return None
    rec["bytes"] = (factor["fetch_factor"] * rec["fetch_kib"] + factor["write_factor"] * rec["write_kib"]) * 1024.0
    return rec


def _time_ms(fn, reps):
    import torch
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    b.synchronize()
    return a.elapsed_time(b) / reps


def epoch_ablation(isp, w, indptr, indices, values, X, dY, epochs):
    """The paper's caching claim at kernel level (Section 3.3): per-epoch time of forward + backward SpMM when
    the transpose is built once and cached vs built again in every epoch.  Both legs run on handles that were
    built beforehand with workspaces that were allocated (and touched) beforehand, so the only work that
    differs between them is the transposition itself: the rebuilt leg uses one fresh handle per epoch, whose
    first isp_csr_transpose_cached call is a cache miss."""
    import torch
    Y, dX = torch.empty_like(X), torch.empty_like(X)
    n, nnz = w.n, w.nnz

    def fresh():
        ws_a = torch.zeros(isp.csr_build_workspace(n, n, nnz), dtype=torch.uint8, device="cuda")
        H = isp.csr_build(indptr, indices, values, workspace=ws_a)
        ws_t = torch.zeros(isp.csr_transpose_workspace(H), dtype=torch.uint8, device="cuda")
        return H, ws_t

    A, ws_t = fresh()

    def epoch_cached():
        isp.spmm(A, X, Y)
        At, _ = isp.csr_transpose_cached(A, workspace=ws_t)  # built in the first epoch only
        isp.spmm(At, dY, dX)

    first = _time_ms(epoch_cached, 1)
    epoch_cached()
    cached = _time_ms(epoch_cached, epochs)

    handles = [fresh() for _ in range(epochs + 1)]
    torch.cuda.synchronize()
    it = iter(handles)

    def epoch_rebuilt():
        B, ws = next(it)
        isp.spmm(B, X, Y)
        Bt, was = isp.csr_transpose_cached(B, workspace=ws)  # a cache miss: the transpose is built here
        assert not was
        isp.spmm(Bt, dY, dX)

    epoch_rebuilt()  # (warm-up on the first spare handle)
    rebuilt = _time_ms(epoch_rebuilt, epochs)
    transpose_ms = rebuilt - cached
    bwd_ms = _time_ms(lambda: isp.spmm(isp.csr_transpose_cached(A)[0], dY, dX), max(3, epochs))
    for B, _ in handles:
        B.destroy()
    return {"what": "epoch ablation: SpMM forward + backward per epoch; handles and workspaces prepared beforehand, "
                    "only the transposition differs", "workload": w.name, "epochs": epochs, "d": w.d,
            "first_epoch_ms_with_cache": round(first, 3), "epoch_ms_cached_transpose": round(cached, 3),
            "epoch_ms_transpose_rebuilt": round(rebuilt, 3), "speedup_from_cache": round(rebuilt / cached, 3),
            "transpose_ms": round(transpose_ms, 3), "backward_spmm_ms": round(bwd_ms, 3),
            # the cache has paid for itself once the epochs' savings exceed nothing at all: the first epoch costs
            # the same either way, every later epoch saves one transposition
            "transpose_cost_in_backward_spmms": round(transpose_ms / bwd_ms, 2), "break_even_epoch": 2}


SWEEP_WIDTHS = (8, 16, 30, 32, 64, 100, 128, 256, 512, 1024)


def sweep_d(isp, w, A, widths=SWEEP_WIDTHS):
    """SpMM forward over feature widths (the GPU counterpart of the paper's tuning graph, Section 3.2),
    including widths that are not multiples of 4 (the narrow-lane kernels) and d = 8."""
    import torch
    out = []
    for d in widths:
        X = torch.randn(w.n, d, device="cuda")
        Y = torch.empty_like(X)
        isp.spmm(A, X, Y)
        ms = _time_ms(lambda: isp.spmm(A, X, Y), 5 if w.nnz > 1 << 22 else 50)
        out.append({"d": d, "ms": round(ms, 4), "gflops": round(2.0 * w.nnz * d / ms / 1e6, 1),
                    "requested_GBps": round(w.nnz * (8.0 + 4.0 * d) / ms / 1e6, 1)})
        del X, Y
    return {"what": "SpMM forward vs feature width; requested_GBps = nnz * (8 + 4 d) bytes over time (every entry "
                    "fetching its own row)", "workload": w.name, "nnz": w.nnz, "sweep": out}


def ceilings(isp):
    """Memory-system ceilings as this path sees them.  (a) A plain device copy (bytes read + written over time).
    (b) The library's SpMM at d = 128 on uniform random graphs (every row 64 random columns, 16 Mi entries)
    whose dense operand X has n_cols rows of 512 bytes: with no skew to exploit, the requested gather bytes
    over time are what random 512-byte row gathers get from wherever a table of that size lives (an XCD's
    4 MB L2, the 256 MB Infinity Cache, HBM)."""
    import numpy as np
    import torch
    out = {"what": "copy and random-row-gather rates by footprint", "copy": [], "gather": []}
    for mb in (8, 64, 256, 1280, 4096):
        n = mb * (1 << 20) // 4
        src = torch.empty(n, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        ms = _time_ms(lambda: dst.copy_(src), 20 if mb <= 256 else 5)
        out["copy"].append({"MB_each_way": mb, "ms": round(ms, 4), "GBps_read_plus_written": round(2.0 * n * 4 / ms / 1e6, 1)})
        del src, dst
    d, deg, n_rows = 128, 64, 1 << 18
    rng = np.random.default_rng(0)
    for mb in (2, 8, 32, 128, 512, 1280):
        n_cols = mb * (1 << 20) // (4 * d)
        cols = np.sort(rng.integers(0, n_cols, size=(n_rows, deg), dtype=np.int64), axis=1).astype(np.int32).reshape(-1)
        indptr = (np.arange(n_rows + 1, dtype=np.int64) * deg)
        A = isp.csr_build(torch.from_numpy(indptr).cuda(), torch.from_numpy(cols).cuda(), None, n_cols=n_cols)
        X = torch.randn(n_cols, d, device="cuda")
        Y = torch.empty(n_rows, d, device="cuda")
        isp.spmm(A, X, Y)
        isp.spmm(A, X, Y)
        ms = _time_ms(lambda: isp.spmm(A, X, Y), 10)
        nnz = n_rows * deg
        out["gather"].append({"X_MB": mb, "columns": n_cols, "entries": nnz, "ms": round(ms, 4),
                              "requested_GBps": round(nnz * 4.0 * d / ms / 1e6, 1),
                              "ps_per_entry": round(ms * 1e9 / nnz, 1)})
        torch.cuda.synchronize()
        A.destroy()
        del X, Y
    return out


def split_rows(isp, w, X, T, reps):
    """SpMM forward on the rows of at most T entries and on the longer rows, each class as a matrix of its own
    (those rows only, all columns), through the library as it is.  The launch on the whole matrix processes the
    two classes one after the other, so the two times say where it goes."""
    import numpy as np
    import torch
    deg = np.diff(w.indptr)
    rows = np.repeat(np.arange(w.n), deg)
    out = []
    for name, keep_row in (("rows <= %d" % T, deg <= T), ("rows > %d" % T, deg > T)):
        keep = keep_row[rows]
        n_sub = int(keep_row.sum())
        ip = np.zeros(n_sub + 1, dtype=np.int64)
        np.cumsum(deg[keep_row], out=ip[1:])
        vals = None if w.values is None else torch.from_numpy(w.values[keep]).cuda()
        H = isp.csr_build(torch.from_numpy(ip).cuda(), torch.from_numpy(w.indices[keep]).cuda(), vals, n_cols=w.n)
        Y = torch.empty(n_sub, w.d, device="cuda")
        isp.spmm(H, X, Y)
        isp.spmm(H, X, Y)
        ms = _time_ms(lambda: isp.spmm(H, X, Y), reps)
        nz = int(keep.sum())
        info = H.info()
        out.append({"class": name, "rows": n_sub, "entries": nz, "ms": round(ms, 4),
                    "ps_per_entry": round(ms * 1e9 / max(nz, 1), 1), "spmm_pieces": info["spmm_pieces"],
                    "work_items": info["spmm_row_blocks"] or info["n_row_blocks"] + info["n_segments"]})
        torch.cuda.synchronize()
        H.destroy()
        del Y
    return {"what": "SpMM forward on the short rows alone and on the long rows alone, each class as a matrix of its own "
                    "(launch order: class 1, then class 2; two warm-up launches each, then %d timed)" % reps,
            "workload": w.name, "d": w.d, "classes": out}


def gcn_step(w, indptr, indices, values, X):
    """End-to-end 2-layer GCN step: out = A relu(A (X W1)) W2, MSE-style loss, backward, SGD update."""
    import torch
    from paper_2403_14853_amd import autograd as ag
    g = ag.SparseGraph(indptr, indices, values)
    d = w.d
    torch.manual_seed(0)
    W1 = (torch.randn(d, d, device="cuda") / d ** 0.5).requires_grad_(True)
    W2 = (torch.randn(d, d, device="cuda") / d ** 0.5).requires_grad_(True)

    def step():
        out = ag.spmm(g, torch.relu(ag.spmm(g, X @ W1)) @ W2)
        loss = out.square().mean()
        loss.backward()
        with torch.no_grad():
            for W in (W1, W2):
                W -= 1e-3 * W.grad
                W.grad = None

    step()
    step()
    ms = _time_ms(step, 10)
    return {"what": "2-layer GCN training step (4 SpMM + 6 GEMM + elementwise)", "workload": w.name, "hidden": d,
            "ms_per_step": round(ms, 3), "sparse_flops": 4 * 2.0 * w.nnz * d,
            "sparse_gflops_if_all_time_were_sparse": round(4 * 2.0 * w.nnz * d / ms / 1e6, 1)}


def reductions(isp, w, A, X, dY):
    """mean / min / max SpMM (generic path) forward and backward, next to the tuned sum."""
    import torch
    Y, dX = torch.empty_like(X), torch.empty_like(X)
    arg = torch.empty(w.n, w.d, dtype=torch.int32, device="cuda")
    out = {}
    for r in ("sum", "mean", "min", "max"):
        a = arg if r in ("min", "max") else None
        isp.spmm_reduce(A, X, Y, r, a)
        f = _time_ms(lambda: isp.spmm_reduce(A, X, Y, r, a), 5)
        isp.spmm_reduce_backward(A, dY, dX, r, a)
        b = _time_ms(lambda: isp.spmm_reduce_backward(A, dY, dX, r, a), 5)
        out[r] = {"forward_ms": round(f, 4), "backward_ms": round(b, 4),
                  "forward_gflops": round(2.0 * w.nnz * w.d / f / 1e6, 1)}
    return {"what": "SpMM reductions, forward and backward through the cached transpose", "workload": w.name,
            "reductions": out}


def cpu_baseline(w, Y_gpu, dom):
    """Time the fp64 CPU oracle on a bounded row sample of the same workload (and use its result
    as one more parity check of the GPU output on those rows)."""
    import numpy as np
    import oracle
    target_nnz = 200_000_000  # whole forward of configs 0-3 (seconds of oracle work on 16 cores)
    rows = int(np.searchsorted(w.indptr, min(target_nnz, w.nnz), side="left"))
    rows = max(1, min(rows, w.n))
    sp = w.indptr[: rows + 1]
    nnz_s = int(sp[-1])
    si, sv = w.indices[:nnz_s], (None if w.values is None else w.values[:nnz_s])
    threads = oracle.max_threads()
    t0 = time.perf_counter()
    if dom == "spmm":
        ref, mag = oracle.spmm(sp, si, sv, w.X, want_mag=True)
        flops, kind = 2.0 * nnz_s * w.d, "spmm forward"
    else:
        ref, mag = oracle.fusedmm(sp, si, sv, w.X, want_mag=True)
        flops, kind = 4.0 * nnz_s * w.d, "fusedmm forward"
    dt = time.perf_counter() - t0
    single = None
    if nnz_s <= 5_000_000:  # small workloads: also the oracle on one thread
        oracle.set_threads(1)
        t1 = time.perf_counter()
        (oracle.spmm if dom == "spmm" else oracle.fusedmm)(sp, si, sv, w.X, want_mag=False)
        single = round(flops / (time.perf_counter() - t1) / 1e9, 2)
        oracle.set_threads(threads)
    got = Y_gpu[:rows].cpu().numpy().astype(np.float64)
    ratio = float(np.max(np.abs(got - ref) / (1e-5 * mag + 1e-6)))
    return {"value": round(flops / dt / 1e9, 2), "unit": "GFLOP/s", "cores": threads, "kind": "oracle",
            "sample": "%s on rows [0, %d) of the same graph (%d stored entries), fp64 accumulate, "
                      "OpenMP over rows, %.1f s" % (kind, rows, nnz_s, dt),
            "single_thread_value": single, "gpu_vs_oracle_max_err_over_tol": ratio}


if __name__ == "__main__":
    main()
