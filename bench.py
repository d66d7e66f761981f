#!/usr/bin/env python3
"""Benchmark of the FTC-GNN hot path on one MI355X.

One step = one pass of the whole hot path on the R-MAT configuration (N = 2^20, ~32.5 M stored
entries, fp16 features N x 128): sparse graph transformation (window build), GCN normalisation,
2-layer GCN forward (128 -> 16 -> 8) and 4-layer AGNN forward (128 -> 32, four propagation
layers, -> 8).  All inputs are resident in HBM before the timed region.

Prints one JSON line.  `value` is the hot path's algorithmic GB/s: the bytes the method has to
move per step (window-deduplicated gathers, every index / value / output once; formulas in
alg_bytes below) divided by the measured step time.  `roofline` is for the dominant kernel, timed
with events on the launch stream inside the timed region.  `cpu_baseline` is the fp64 oracle
running the same pass on a smaller R-MAT graph of the same recipe on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def alg_bytes(n, nnz, sum_uniq, n_win):
    """Algorithmic bytes of every call of one step, keyed by call name."""
    e = 2  # fp16 activations
    rp = 4 * (n + 1)
    b = {}
    b["build_windows"] = nnz * 4 + rp + nnz * 8 + sum_uniq * 4 + n_win * 8
    b["gcn_norm"] = rp + n * 4   # factored normalisation: only dinv[n] is produced, no per-edge values

    def gemm(di, do, o, scaled=False):
        return n * di * e + di * do * e + n * do * o + (n * 4 if scaled else 0)

    def spmm(d, e_in, o):
        # column index per edge, no edge values (the GCN layers use dinv), dinv[n] for the output scale
        return sum_uniq * d * e_in + nnz * 4 + n * d * o + n * 4 + rp

    def sddmm(d):
        return sum_uniq * d * e + n * d * e + nnz * 8 + rp

    # GCN layer = update GEMM (fp16 Z, rows scaled by dinv) + aggregation over Z
    b["gcn_l1_gemm"] = gemm(128, 16, 2, True)
    b["gcn_l1_spmm"] = spmm(16, 2, 2)
    b["gcn_l2_gemm"] = gemm(16, 8, 2, True)
    b["gcn_l2_spmm"] = spmm(8, 2, 4)
    b["agnn_in_gemm"] = gemm(128, 32, 2)
    for l in range(4):
        # fused propagation layer: one gather per condensed column, own rows once, column index once,
        # output once (the row norms are recomputed from the rows in registers)
        b[f"agnn_l{l}_fused"] = sum_uniq * 32 * e + n * 32 * e + nnz * 4 + n * 32 * 2
    b["agnn_out_gemm"] = gemm(32, 8, 4)
    return b


def cpu_baseline(scale, seed, g=None):
    """The oracle's whole hot path on an R-MAT graph of 2^scale nodes; returns the dict for the JSON."""
    import numpy as np
    import synth
    from oracle import ftc_oracle as orc
    if g is None:
        g = synth.rmat(scale, 16, seed)
    rng_x = synth.normal_features(g.n, 128, seed + 10).astype(np.float16).astype(np.float64)
    W1 = synth.glorot_uniform(128, 16, seed + 11).astype(np.float64)
    W2 = synth.glorot_uniform(16, 8, seed + 12).astype(np.float64)
    Win = synth.glorot_uniform(128, 32, seed + 13).astype(np.float64)
    Wout = synth.glorot_uniform(32, 8, seed + 14).astype(np.float64)
    threads = orc.set_threads(0)
    t0 = time.perf_counter()
    win = orc.build_windows(g.row_ptr, g.col_idx)
    vals, _ = orc.gcn_norm(g.row_ptr, g.col_idx)
    h, _ = orc.gcn_layer(g.row_ptr, g.col_idx, vals, rng_x, W1, relu=True)
    orc.gcn_layer(g.row_ptr, g.col_idx, vals, h, W2)
    a, _ = orc.gemm(rng_x, Win)
    a = np.maximum(a, 0)
    for _ in range(4):
        a, _, _ = orc.agnn_layer(g.row_ptr, g.col_idx, a, 1.0)
    orc.gemm(a, Wout)
    dt = time.perf_counter() - t0
    orc.set_threads(1)
    total = sum(alg_bytes(g.n, g.nnz, int(win["summary"][0]), win["n_windows"]).values())
    return {"value": total / dt / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"whole hot path on R-MAT scale {scale} ({g.n} nodes, {g.nnz} stored entries), "
                      f"same recipe as the workload, {dt:.1f} s"}


def fabric_bytes(key):
    """Counter-measured L2 <-> fabric bytes per launch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy of
    known size) from the committed summary; None where no profile covers the kernel."""
    path = os.path.join(ROOT, "profiles", "fabric_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        return json.load(f).get(key)


def kernel_suite(tag, g, feat32, dtype, D, iters=20, oracle=False, ops=("spmm", "sddmm", "softmax")):
    """Stand-alone SpMM / SDDMM / edge-softmax timings on one graph (events on the launch stream), warm (back to
    back) and cold (a 1 GiB buffer is overwritten between launches).  Per operation three byte counts: `alg`
    (what the method moves: one gathered row per distinct window column, every index / value / output once),
    `compulsory` (every array once: the lower bound no access order can beat) and `fabric` (what the counters
    saw between L2 and the fabric; reads served by the memory-side cache count there as well as reads from HBM)."""
    import numpy as np
    import torch
    from paper_2412_12218_amd import binding as B
    dev = torch.device("cuda:0")
    dg = B.Graph.from_numpy(g.row_ptr, g.col_idx)
    win = B.ftc_build_windows(dg)
    vals, _ = B.ftc_gcn_norm(dg, win)
    X = torch.from_numpy(feat32).to(dtype).to(dev)
    out = torch.empty((g.n, D), dtype=torch.float32, device=dev)
    s_out = torch.empty(g.nnz, dtype=torch.float32, device=dev)
    ws = B._workspace(max(B.lib().ftc_spmm_workspace_bytes(g.n, g.nnz, D),
                          B.lib().ftc_sddmm_workspace_bytes(g.n, g.nnz, D)), dev)
    flush = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    sum_uniq = int(win.summary[0].item())
    e = X.element_size()
    rp = 4 * (g.n + 1)
    nbytes = {"spmm": sum_uniq * D * e + g.nnz * 8 + g.n * D * 4 + rp,
              "sddmm": sum_uniq * D * e + g.n * D * e + g.nnz * 8 + rp,
              "softmax": g.nnz * 8 + rp}
    compulsory = {"spmm": g.n * D * e + g.nnz * 8 + g.n * D * 4 + rp,     # X, column ids + values, output, row starts
                  "sddmm": g.n * D * e + g.nnz * 8 + rp,                  # X (= Y), column ids + scores, row starts
                  "softmax": g.nnz * 8 + rp}
    ws_sm = B._workspace(B.lib().ftc_edge_softmax_workspace_bytes(g.n, g.nnz), dev)
    p_out = torch.empty(g.nnz, dtype=torch.float32, device=dev)
    fns = {"spmm": lambda: B.ftc_spmm(dg, win, vals, X, out=out, ws=ws),
           # edge scores of AGNN: beta * cos(h_i, h_j), norms recomputed from the gathered rows
           "sddmm": lambda: B.ftc_sddmm(dg, win, X, X, None, None, 1.0, out=s_out, ws=ws, cosine=True),
           # edge softmax over the scores the SDDMM has just written
           "softmax": lambda: B.ftc_edge_softmax(dg, win, s_out, out=p_out, ws=ws_sm)}
    res = {"graph": tag, "n": g.n, "nnz": g.nnz, "sum_uniq": sum_uniq, "D": D, "dtype": str(dtype)[6:],
           "feature_matrix_MB": g.n * D * e / 1e6}
    for op, fn in fns.items():
        if op not in ops:
            continue
        for _ in range(5):
            fn()
        for mode in ("warm", "cold"):
            ts = []
            for _ in range(iters):
                if mode == "cold":
                    flush.zero_()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                fn()
                b.record()
                b.synchronize()
                ts.append(a.elapsed_time(b))
            ms = float(np.mean(ts))
            res[f"{op}_{mode}_ms"] = ms
            res[f"{op}_{mode}_min_ms"] = float(np.min(ts))
            res[f"{op}_{mode}_GBs"] = nbytes[op] / (ms * 1e-3) / 1e9
            res[f"{op}_{mode}_frac"] = nbytes[op] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
        res[f"{op}_alg_bytes"] = nbytes[op]
        res[f"{op}_compulsory_bytes"] = compulsory[op]
        res[f"{op}_fabric_bytes"] = fabric_bytes(f"{tag.split()[0]}_D{D}_{op}")
    if oracle:
        del X, out, s_out, p_out, flush, ws, ws_sm
        res["oracle"] = oracle_kernel_times(g, feat32, dtype, nbytes)
    return res


def oracle_kernel_times(g, feat32, dtype, nbytes):
    """The oracle's SpMM / SDDMM (cosine scores) / edge softmax on the same graph and the same quantised
    features, one thread and all host threads: seconds and GB/s by the same algorithmic byte counts."""
    import numpy as np
    import torch
    from oracle import ftc_oracle as orc
    X = torch.from_numpy(feat32).to(dtype).to(torch.float64).numpy()
    vals, _ = orc.gcn_norm(g.row_ptr, g.col_idx)
    rinv = orc.row_rnorm(X)
    s = orc.sddmm(g.row_ptr, g.col_idx, X, X, rinv, rinv, 1.0)
    fns = {"spmm": lambda: orc.spmm(g.row_ptr, g.col_idx, vals, X),
           "sddmm": lambda: orc.sddmm(g.row_ptr, g.col_idx, X, X, rinv, rinv, 1.0),
           "softmax": lambda: orc.edge_softmax(g.row_ptr, s)}
    res = {}
    orc.set_threads(0)
    for fn in fns.values():     # untimed: thread pool start-up, first touch of the allocator's pages
        fn()
    for label, t in (("1_thread", 1), ("all_threads", 0)):
        used = orc.set_threads(t)
        for op, fn in fns.items():
            t0 = time.perf_counter()
            fn()
            dt = time.perf_counter() - t0
            res[f"{op}_{label}_s"] = dt
            res[f"{op}_{label}_GBs"] = nbytes[op] / dt / 1e9
        res[f"{label}_count"] = used
    orc.set_threads(1)
    return res


def density_sweep(n=1 << 18, k=32, dims=(32, 64, 128, 256), iters=20):
    """Vector path vs matrix-core path on graphs whose 16-row windows have a controlled reuse of
    gathered rows (edges per condensed column = 16 k / pool).  Prints one JSON line per point."""
    import numpy as np
    import torch
    import synth
    from paper_2412_12218_amd import binding as B
    dev = torch.device("cuda:0")

    def avg_ms(fn):
        for _ in range(3):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        b.synchronize()
        return a.elapsed_time(b) / iters

    for pool in (512, 384, 256, 192, 128, 96, 64, 48, 32):
        g = synth.fill_controlled(n, pool, k, seed=5)
        dg = B.Graph.from_numpy(g.row_ptr, g.col_idx)
        win = B.ftc_build_windows(dg)
        sum_uniq = int(win.summary[0].item())
        vals = torch.rand(g.nnz, dtype=torch.float32, device=dev)
        for D in dims:
            X = torch.from_numpy(synth.normal_features(g.n, D, 6)).to(torch.float16).to(dev)
            out = torch.empty((g.n, D), dtype=torch.float32, device=dev)
            s_out = torch.empty(g.nnz, dtype=torch.float32, device=dev)
            ws = B._workspace(B.lib().ftc_spmm_workspace_bytes(g.n, g.nnz, D), dev)
            rec = {"pool": pool, "reuse": g.nnz / sum_uniq, "tile_fill": g.nnz / (16.0 * sum_uniq), "D": D,
                   "nnz": g.nnz}
            for name, path in (("valu", B.FTC_PATH_VALU), ("mfma", B.FTC_PATH_MFMA)):
                rec[f"spmm_{name}_ms"] = avg_ms(lambda: B.ftc_spmm(dg, win, vals, X, out=out, path=path, ws=ws))
                rec[f"sddmm_{name}_ms"] = avg_ms(lambda: B.ftc_sddmm(dg, win, X, X, None, None, 1.0, out=s_out,
                                                                      path=path, ws=ws))
            print(json.dumps(rec), flush=True)


def reorder_suite(iters=10):
    """What the locality reordering costs and what it buys: per benchmark graph and ordering, the time
    of ftc_degree_order + ftc_permute_graph, the share of distinct window columns (sum_uniq / nnz) and
    the aggregation kernels before and after.  One JSON line per (graph, ordering)."""
    import torch
    import synth
    from paper_2412_12218_amd import binding as B
    dev = torch.device("cuda:0")

    def ms_of(fn, reps=iters):
        for _ in range(2):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        b.synchronize()
        return a.elapsed_time(b) / reps

    def kernels(dg, D, dtype):
        win = B.ftc_build_windows(dg)
        X = torch.randn(dg.n, D, device=dev).to(dtype)
        X16 = torch.randn(dg.n, 16, device=dev).to(torch.float16)
        out = torch.empty(dg.n, D, device=dev)
        out16 = torch.empty(dg.n, 16, device=dev)
        outh = torch.empty(dg.n, D, device=dev, dtype=dtype)
        sc = torch.empty(dg.nnz, device=dev)
        L = B.lib()
        ws = B._workspace(max(L.ftc_agnn_layer_workspace_bytes(dg.n, dg.nnz, D), L.ftc_spmm_workspace_bytes(dg.n, dg.nnz, D),
                              L.ftc_sddmm_workspace_bytes(dg.n, dg.nnz, D)), dev)
        return {"uniq_per_nnz": int(win.summary[0].item()) / max(dg.nnz, 1),
                "spmm_ms": ms_of(lambda: B.ftc_spmm(dg, win, None, X, out=out, ws=ws)),
                "spmm_d16_ms": ms_of(lambda: B.ftc_spmm(dg, win, None, X16, out=out16, ws=ws)),
                "sddmm_cos_ms": ms_of(lambda: B.ftc_sddmm(dg, win, X, X, None, None, 1.0, out=sc, ws=ws, cosine=True)),
                "agnn_fused_ms": ms_of(lambda: B.ftc_agnn_layer(dg, win, X, out=outh, ws=ws))}

    for cfg, D, dtype in ((5, 32, torch.float16), (4, 64, torch.bfloat16), (3, 32, torch.float16), (2, 32, torch.float16)):
        g = synth.config_graph(cfg)
        dg = B.Graph.from_numpy(g.row_ptr, g.col_idx)
        base = kernels(dg, D, dtype)
        stats = B.ftc_degree_stats(dg).cpu().numpy()
        plan = B.ftc_plan_graph(g.n, g.nnz, int(stats[0]), int(round(base["uniq_per_nnz"] * g.nnz)), D, dtype)
        print(json.dumps({"graph": f"cfg{cfg}", "n": g.n, "nnz": g.nnz, "D": D, "ordering": "as given", **base,
                          "plan": plan}), flush=True)
        ws = B._workspace(B.lib().ftc_reorder_workspace_bytes(g.n, g.nnz), dev)
        for mode, tag in ((B.FTC_ORDER_DEGREE, "degree"), (B.FTC_ORDER_DEGREE_CLASSES, "degree classes"),
                          (None, "communities (10 rounds of label propagation)")):
            if mode is None:
                order = lambda: B.ftc_order_by_key(B.ftc_label_propagation(dg, 10, ws=ws), ws=ws)[:2]
            else:
                order = lambda: B.ftc_degree_order(dg, mode, ws=ws)
            t_order = ms_of(order, 3)
            perm, inv = order()
            t_graph = ms_of(lambda: B.ftc_permute_graph(dg, perm, inv, ws=ws), 5)
            pg, flag = B.ftc_permute_graph(dg, perm, inv, ws=ws)
            assert int(flag.item()) == 0
            Xf = torch.randn(g.n, D, device=dev).to(dtype)
            t_rows = ms_of(lambda: B.ftc_permute_rows(Xf, perm))
            r = kernels(pg, D, dtype)
            print(json.dumps({"graph": f"cfg{cfg}", "ordering": tag, "ordering_ms": t_order, "permute_graph_ms": t_graph,
                              "permute_rows_ms": t_rows, **r}), flush=True)
            del pg, perm, inv
        del dg, ws


def train_suite(scale, iters=10):
    """Forward + backward of the two benchmark models on the benchmark graph (TrainPath): per-call
    times from events on the launch stream.  Prints one JSON line of its own; the benchmark metric
    stays the forward hot path."""
    import numpy as np
    import torch
    import synth
    from paper_2412_12218_amd import binding as B
    from paper_2412_12218_amd.models import TrainPath
    dev = torch.device("cuda:0")
    seed = synth.CONFIGS[5]["seed"]
    g = synth.rmat(scale, 16, seed)
    dg = B.Graph.from_numpy(g.row_ptr, g.col_idx)
    win = B.ftc_build_windows(dg)
    _, dinv = B.ftc_gcn_norm(dg, win, want_vals=False)
    h16 = lambda a: torch.from_numpy(a).to(torch.float16).to(dev)
    X = h16(synth.normal_features(g.n, 128, seed + 10))
    W1, W2 = h16(synth.glorot_uniform(128, 16, seed + 11)), h16(synth.glorot_uniform(16, 8, seed + 12))
    Win, Wout = h16(synth.glorot_uniform(128, 32, seed + 13)), h16(synth.glorot_uniform(32, 8, seed + 14))
    H0 = h16(synth.normal_features(g.n, 32, seed + 20))
    d_gcn = torch.from_numpy(synth.normal_features(g.n, 8, seed + 21)).to(dev)
    d_agnn = h16(synth.normal_features(g.n, 32, seed + 22))
    betas = [1.0] * 4
    times = {}

    def timed(name, fn):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        r = fn()
        b.record()
        b.synchronize()
        times.setdefault(name, []).append(a.elapsed_time(b))
        return r

    for it in range(iters + 2):
        if it == 2:
            times.clear()
        timed("transpose_index", lambda: B.ftc_transpose_index(dg, win))
    tp = TrainPath(dg, win, dinv)
    for it in range(iters + 2):
        if it == 2:
            keep = times.pop("transpose_index")
            times.clear()
            times["transpose_index"] = keep
        timed("gcn_forward_2layers", lambda: tp.gcn_forward(X, W1, W2))
        timed("gcn_backward_2layers", lambda: tp.gcn_backward(X, W1, W2, d_gcn))
        timed("agnn_forward_4layers_keeping_row_z_and_fp32_output", lambda: tp.agnn_forward(H0, betas))
        timed("agnn_backward_4layers", lambda: tp.agnn_backward(betas, d_agnn))
        timed("agnn_model_forward", lambda: tp.agnn_model_forward(X, Win, Wout, betas))
        timed("agnn_model_backward", lambda: tp.agnn_model_backward(X, Win, Wout, betas, d_gcn))
    print(json.dumps({"workload": f"cfg5 R-MAT scale {scale}: N={g.n}, nnz={g.nnz}, fp16 activations, fp32 gradients "
                                  "of weights, GCN 128-16-8, AGNN 32 x 4 layers",
                      "ms": {k: float(np.mean(v)) for k, v in times.items()}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--scale", type=int, default=20, help="R-MAT scale (20 = the benchmark workload)")
    ap.add_argument("--cpu-scale", type=int, default=20, help="R-MAT scale of the oracle's sample; 0 = skip")
    ap.add_argument("--no-kernels", action="store_true", help="skip the stand-alone SpMM/SDDMM section")
    ap.add_argument("--no-reordered", action="store_true", help="skip the step on the relabelled graph")
    ap.add_argument("--reorder", action="store_true",
                    help="instead of the benchmark: cost and effect of the locality reordering on the benchmark graphs")
    ap.add_argument("--train", action="store_true",
                    help="instead of the benchmark: forward + backward times of the two models on the benchmark graph")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark: vector vs matrix-core path over window density")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives or sharding are part of it); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth
    from paper_2412_12218_amd import binding as B
    from paper_2412_12218_amd.models import HotPath

    B.lib()
    if args.sweep:
        density_sweep()
        return
    if args.train:
        train_suite(args.scale)
        return
    if args.reorder:
        reorder_suite()
        return
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    seed = synth.CONFIGS[5]["seed"]
    t0 = time.perf_counter()
    g = synth.rmat(args.scale, 16, seed)
    X = torch.from_numpy(synth.normal_features(g.n, 128, seed + 10)).to(torch.float16).to(dev)
    W1 = torch.from_numpy(synth.glorot_uniform(128, 16, seed + 11)).to(torch.float16).to(dev)
    W2 = torch.from_numpy(synth.glorot_uniform(16, 8, seed + 12)).to(torch.float16).to(dev)
    Win = torch.from_numpy(synth.glorot_uniform(128, 32, seed + 13)).to(torch.float16).to(dev)
    Wout = torch.from_numpy(synth.glorot_uniform(32, 8, seed + 14)).to(torch.float16).to(dev)
    betas = [1.0] * 4
    dg = B.Graph.from_numpy(g.row_ptr, g.col_idx)
    hp = HotPath(dg)
    gen_s = time.perf_counter() - t0

    for _ in range(args.warmup):
        hp.step(X, W1, W2, Win, Wout, betas)
    torch.cuda.synchronize()
    sum_uniq = int(hp.win.summary[0].item())
    bytes_by_call = alg_bytes(g.n, g.nnz, sum_uniq, hp.win.n_windows)
    total_bytes = sum(bytes_by_call.values())

    # Events on the launch stream.  Inside the timed region only the dominant call (ftc_agnn_layer, four per
    # step) is bracketed: its average duration is the roofline's denominator.  The breakdown over all calls
    # comes from extra steps after the timed region (every event pair costs a few microseconds of stream time).
    calls = []
    L = B.lib()
    C = B.C

    def one_step(bracket_all):
        def timed(name, fn):
            if not (bracket_all or name == "agnn_layer"):
                fn()
                return
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            calls.append((name, a, b, bracket_all))

        timed("build_windows", lambda: B.ftc_build_windows_concurrent(dg, hp.side, out=hp.win, ws=hp.ws_win))
        timed("gcn_norm", lambda: B._check(L.ftc_gcn_norm(
            C.byref(dg.c), C.byref(hp.win.c), None, B._ptr(hp.dinv), B._stream())))
        timed("gcn_layer1", lambda: B.ftc_gcn_layer(dg, hp.win, None, X, W1, relu=True, out=hp.gcn_h, ws=hp.ws,
                                                    dinv=hp.dinv))
        timed("gcn_layer2", lambda: B.ftc_gcn_layer(dg, hp.win, None, hp.gcn_h, W2, out=hp.gcn_out, ws=hp.ws,
                                                    dinv=hp.dinv))
        a, b = hp.agnn_h
        timed("agnn_in_gemm", lambda: B.ftc_update_gemm(X, Win, out=a, relu=True))
        for l in range(4):
            timed("agnn_layer", lambda: B.ftc_agnn_layer(dg, hp.win, a, beta=betas[l], out=b, ws=hp.ws))
            a, b = b, a
        timed("agnn_out_gemm", lambda: B.ftc_update_gemm(a, Wout, out=hp.agnn_out))

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step(False)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    for _ in range(3):           # untimed: the per-call breakdown
        one_step(True)
    torch.cuda.synchronize()

    per_call, dominant = {}, []
    for name, a, b, breakdown in calls:
        if breakdown:
            per_call.setdefault(name, []).append(a.elapsed_time(b))
        else:
            dominant.append(a.elapsed_time(b))      # agnn_layer inside the timed region
    avg_ms = {k: float(np.mean(v)) for k, v in per_call.items()}
    avg_ms["agnn_layer"] = float(np.mean(dominant))
    # dominant kernel of the step: the fused AGNN propagation kernel (four launches per step); its
    # call also runs the small fix-up kernel for rows cut by wave ranges, which is included in the time
    dom = "agnn_layer"
    dom_bytes = bytes_by_call["agnn_l0_fused"]
    dom_gbs = dom_bytes / (avg_ms[dom] * 1e-3) / 1e9
    out = {
        "metric": "hot-path algorithmic GB/s (window build + GCN norm + 2-layer GCN + 4-layer AGNN forward)",
        "value": total_bytes / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"cfg5 R-MAT scale {args.scale}: N={g.n}, nnz={g.nnz}, sum_uniq={sum_uniq}, "
                               "fp16 features Nx128, GCN 128-16-8, AGNN 128-32x4-8, fp32 accumulate"},
        "roofline": {"bound": "hbm", "kernel": "agnn_fused_kernel + agnn_fused_fixup_kernel (call ftc_agnn_layer)", "achieved": dom_gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dom_gbs / HBM_PEAK_GBS, "traffic": None,
                     "traffic_kind": "bytes between L2 and the fabric per launch (FETCH_SIZE x 2 + WRITE_SIZE); the 64 MB "
                                     "feature matrix fits the memory-side cache, so most of these reads never reach HBM",
                     "alg_bytes_per_launch": dom_bytes, "avg_ms": avg_ms[dom]},
        "gcn_2layer_ms": avg_ms["gcn_layer1"] + avg_ms["gcn_layer2"],
        "agnn_layer_ms": avg_ms["agnn_layer"],
        "build_windows_ms": avg_ms["build_windows"],
        "call_ms": avg_ms,
        "alg_bytes_per_step": total_bytes,
        "input_generation_s": gen_s,
    }
    # one plain device-to-device copy of known size (1 GiB read + 1 GiB written, far larger than any
    # cache): the reference dispatch against which the profiler's FETCH_SIZE / WRITE_SIZE counters
    # are scaled
    calib_src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
    calib_dst = torch.empty_like(calib_src)
    calib_dst.copy_(calib_src)
    torch.cuda.synchronize()
    del calib_src, calib_dst
    # L2 <-> fabric traffic of the dominant kernel from the committed counter summary (separate profiler runs)
    out["roofline"]["traffic"] = fabric_bytes("cfg5_agnn_fused_kernel")
    if out["roofline"]["traffic"]:
        out["roofline"]["achieved_by_traffic"] = out["roofline"]["traffic"] / (avg_ms[dom] * 1e-3) / 1e9
    # the same step captured once as a HIP graph and replayed (one launch per step instead of ~45)
    graph = hp.capture(X, W1, W2, Win, Wout, betas)
    for _ in range(args.warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    out["graph_replay_ms_per_step"] = (time.perf_counter() - t0) / args.steps * 1e3
    del graph
    if not args.no_reordered:
        # the same step on the graph as the per-graph plan prepares it (statistics -> ftc_plan_graph -> relabelling;
        # one-time preprocessing, timed separately): reported beside the benchmark value, which stays the graph as given
        from paper_2412_12218_amd.models import PlannedGraph
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        pl = PlannedGraph(dg, 32, torch.float16, side=hp.side)
        Xp = pl.enter(X)
        torch.cuda.synchronize()
        prep_ms = (time.perf_counter() - t0) * 1e3
        hp2 = HotPath(pl.g)
        for _ in range(args.warmup):
            hp2.step(Xp, W1, W2, Win, Wout, betas)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            hp2.step(Xp, W1, W2, Win, Wout, betas)
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - t0) / args.steps * 1e3
        out["reordered"] = {"plan": pl.plan, "applied": pl.applied,
                            "preprocessing_ms": prep_ms, "ms_per_step": ms2, "sum_uniq": pl.sum_uniq,
                            "speedup_vs_as_given": ms_per_step / ms2,
                            "break_even_steps": prep_ms / (ms_per_step - ms2) if ms2 < ms_per_step else None}
        del hp2, pl, Xp
    if not args.no_kernels:
        # the two largest graphs: stand-alone aggregation and edge-score kernels, fp32 output
        k5 = kernel_suite("cfg5 R-MAT", g, synth.normal_features(g.n, 32, seed + 20), torch.float16, 32,
                          oracle=args.cpu_scale > 0)
        g4 = synth.config_graph(4) if args.scale == 20 else synth.config_graph(4, 2.0 ** (args.scale - 20))
        k4 = kernel_suite("cfg4 SBM", g4, synth.uniform_features(g4.n, 64, 3 + 20), torch.bfloat16, 64,
                          oracle=args.cpu_scale > 0)
        # the same graph with a feature matrix of 512 MB, twice the memory-side cache: what the gather kernels do
        # when the rows have to come from HBM
        k4big = kernel_suite("cfg4 SBM", g4, synth.uniform_features(g4.n, 256, 3 + 21), torch.bfloat16, 256,
                             ops=("spmm", "sddmm"))
        out["kernels"] = [k4, k5, k4big]
    if args.cpu_scale > 0:
        out["cpu_baseline"] = cpu_baseline(args.cpu_scale, seed, g if args.cpu_scale == args.scale else None)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
