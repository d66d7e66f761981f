"""GPU parity at the full benchmark sizes (configurations 2-5), through the same calls and
buffers that bench.py times (paper_2412_12218_amd.models.HotPath for the R-MAT workload).
The C oracle is fast enough to check every output element; the whole file takes a few minutes,
most of it generating the graphs and running the oracle on the host."""
import numpy as np
import pytest
import torch

import synth
from parity import TOL, check_windows, dev_graph, norm_err, quantise
from paper_2412_12218_amd import binding as B
from paper_2412_12218_amd.models import HotPath, PlannedGraph

pytestmark = pytest.mark.gpu
F32, F16, BF16 = torch.float32, torch.float16, torch.bfloat16


def say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def threads(oracle):
    t = oracle.set_threads(0)
    yield t
    oracle.set_threads(1)


def factored_vals(g, oracle):
    """fp32 dinv of the oracle and the fp64 products dinv[i] * dinv[j] of those fp32 numbers."""
    _, dinv64 = oracle.gcn_norm(g.row_ptr, g.col_idx)
    dinv32 = dinv64.astype(np.float32)
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    return dinv32, dinv32[rows].astype(np.float64) * dinv32[g.col_idx].astype(np.float64)


def test_cfg2_gcn_layer_full(oracle, threads):
    g = synth.config_graph(2)
    say(f"cfg2 n={g.n} nnz={g.nnz}")
    vals64, _ = oracle.gcn_norm(g.row_ptr, g.col_idx)
    vals32 = vals64.astype(np.float32)
    Xd, X64 = quantise(synth.uniform_features(g.n, 128, seed=1), F16)
    Wd, W64 = quantise(synth.glorot_uniform(128, 32, seed=1), F16)
    ref, ab = oracle.gcn_layer(g.row_ptr, g.col_idx, vals32.astype(np.float64), X64, W64)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    check_windows(win, oracle.build_windows(g.row_ptr, g.col_idx))
    vals_gpu, _ = B.ftc_gcn_norm(dg, win)
    assert np.max(np.abs(vals_gpu.cpu().double().numpy() - vals64) / vals64) < 1e-6
    out = B.ftc_gcn_layer(dg, win, torch.from_numpy(vals32).cuda(), Xd, Wd)
    err = norm_err(out, ref, ab)
    say(f"  gcn_layer err {err:.3e}")
    assert err < 2e-3
    # factored normalisation (dinv instead of per-edge values)
    dinv32, fvals64 = factored_vals(g, oracle)
    ref, ab = oracle.gcn_layer(g.row_ptr, g.col_idx, fvals64, X64, W64)
    out = B.ftc_gcn_layer(dg, win, None, Xd, Wd, dinv=torch.from_numpy(dinv32).cuda())
    err = norm_err(out, ref, ab)
    say(f"  gcn_layer (factored) err {err:.3e}")
    assert err < 2e-3


def test_cfg3_agnn_layer_full(oracle, threads):
    g = synth.config_graph(3)
    say(f"cfg3 n={g.n} nnz={g.nnz}")
    Hd, H64 = quantise(synth.normal_features(g.n, 32, seed=2), F16)
    ref, ab, pref = oracle.agnn_layer(g.row_ptr, g.col_idx, H64, 1.0)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    out = B.ftc_agnn_layer(dg, win, Hd, beta=1.0)
    err = norm_err(out, ref, ab)
    p = torch.empty(g.nnz, dtype=F32, device="cuda")
    out_u = B.ftc_agnn_layer(dg, win, Hd, beta=1.0, edge_p=p)
    err_u = norm_err(out_u, ref, ab)
    perr = float(np.max(np.abs(p.cpu().double().numpy() - pref) / pref))
    say(f"  fused err {err:.3e}, unfused err {err_u:.3e}, p err {perr:.3e}")
    assert err < 2e-3 and err_u < 2e-3 and perr < 2e-3


def test_cfg4_spmm_sddmm_full(oracle, threads):
    g = synth.config_graph(4)
    say(f"cfg4 n={g.n} nnz={g.nnz}")
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    torch.cuda.synchronize()
    check_windows(win, oracle.build_windows(g.row_ptr, g.col_idx))
    say("  window index bit-exact")
    vals64, _ = oracle.gcn_norm(g.row_ptr, g.col_idx)
    vals32 = vals64.astype(np.float32)
    Xd, X64 = quantise(synth.uniform_features(g.n, 64, seed=3), BF16)
    ref, ab = oracle.spmm(g.row_ptr, g.col_idx, vals32.astype(np.float64), X64)
    out = B.ftc_spmm(dg, win, torch.from_numpy(vals32).cuda(), Xd)
    err = norm_err(out, ref, ab)
    say(f"  spmm err {err:.3e}")
    assert err < 2e-3
    del ref, ab, out
    rinv64 = oracle.row_rnorm(X64)
    rinv = B.ftc_row_rnorm(Xd)
    assert np.max(np.abs(rinv.cpu().double().numpy() - rinv64) / rinv64) < 1e-5
    rinv32 = rinv64.astype(np.float32)
    sref, sab = oracle.sddmm(g.row_ptr, g.col_idx, X64, X64, rinv32.astype(np.float64), rinv32.astype(np.float64), 1.0)
    s = B.ftc_sddmm(dg, win, Xd, Xd, torch.from_numpy(rinv32).cuda(), torch.from_numpy(rinv32).cuda(), 1.0)
    serr = norm_err(s, sref, sab)
    say(f"  sddmm err {serr:.3e}")
    assert serr < 2e-3
    # the call bench.py times: cosine mode, norms recomputed in the kernel
    sref, sab = oracle.sddmm(g.row_ptr, g.col_idx, X64, X64, rinv64, rinv64, 1.0)
    s = B.ftc_sddmm(dg, win, Xd, Xd, cosine=True)
    serr = norm_err(s, sref, sab)
    say(f"  sddmm (cosine) err {serr:.3e}")
    assert serr < 2e-3


def test_cfg4_wide_features_sampled_rows(oracle, threads):
    """The benchmark's out-of-cache point: cfg4 with a 512 MB feature matrix (bf16, D = 256).  The kernels run on the
    whole graph; the oracle computes 40 000 sampled rows (a sub-matrix of those rows with all columns kept) and every
    one of their elements and entries is compared."""
    g = synth.config_graph(4)
    D = 256
    say(f"cfg4 D={D} n={g.n} nnz={g.nnz}")
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    vals64, _ = oracle.gcn_norm(g.row_ptr, g.col_idx)
    vals32 = vals64.astype(np.float32)
    Xd, X64 = quantise(synth.uniform_features(g.n, D, seed=4), BF16)
    out = B.ftc_spmm(dg, win, torch.from_numpy(vals32).cuda(), Xd)
    s = B.ftc_sddmm(dg, win, Xd, Xd, cosine=True)
    torch.cuda.synchronize()
    rng = np.random.default_rng(44)
    rows = np.sort(rng.choice(g.n, size=40_000, replace=False))
    rows[:3] = [0, 1, 2]
    rows[-1] = g.n - 1
    rows = np.unique(rows)
    rp = g.row_ptr.astype(np.int64)
    deg = (rp[rows + 1] - rp[rows])
    sub_ptr = np.zeros(rows.size + 1, dtype=np.int64)
    sub_ptr[1:] = np.cumsum(deg)
    entries = np.concatenate([np.arange(rp[r], rp[r + 1]) for r in rows])
    sub_col = g.col_idx[entries]
    # SpMM of the sampled rows: a matrix with those rows and all n columns
    ref, ab = oracle.spmm(sub_ptr.astype(np.int32), sub_col, vals32[entries].astype(np.float64), X64)
    err = norm_err(out[torch.from_numpy(rows).cuda()], ref, ab)
    say(f"  spmm err on {rows.size} rows {err:.3e}")
    assert err < 2e-3
    # cosine scores of their entries: x_i is row rows[k] of X
    rinv64 = oracle.row_rnorm(X64)
    Xrows = X64[rows]
    dots = np.empty(entries.size)
    dabs = np.empty(entries.size)
    pos = 0
    for k in range(rows.size):
        c = sub_col[sub_ptr[k]:sub_ptr[k + 1]]
        prod = X64[c] * Xrows[k]
        dots[pos:pos + c.size] = prod.sum(axis=1) * rinv64[rows[k]] * rinv64[c]
        dabs[pos:pos + c.size] = np.abs(prod).sum(axis=1) * rinv64[rows[k]] * rinv64[c]
        pos += c.size
    serr = norm_err(s[torch.from_numpy(entries).cuda()], dots, dabs)
    say(f"  sddmm (cosine) err on {entries.size} entries {serr:.3e}")
    assert serr < 2e-3


def test_cfg5_planned_graph_agnn_layer_full(oracle, threads):
    """The benchmark's relabelled leg at full size: the per-graph plan (degree classes on the R-MAT workload), one
    AGNN layer on the relabelled graph, features in and results out through the permutations, every element against
    the oracle on the graph as given."""
    g = synth.config_graph(5)
    dg = dev_graph(g)
    pg = PlannedGraph(dg, 32, F16)
    say(f"cfg5 plan applied: {pg.applied}, sum_uniq {pg.sum_uniq} (given {pg.sum_uniq_given})")
    assert pg.applied == "degree classes" and pg.sum_uniq < pg.sum_uniq_given
    Hd, H64 = quantise(synth.normal_features(g.n, 32, seed=55), F16)
    ref, ab, _ = oracle.agnn_layer(g.row_ptr, g.col_idx, H64, 1.0)
    out = pg.leave(B.ftc_agnn_layer(pg.g, pg.win, pg.enter(Hd), beta=1.0))
    err = norm_err(out, ref, ab)
    say(f"  agnn_layer through the plan err {err:.3e}")
    assert err < 2e-3


def test_cfg5_models_layer_by_layer(oracle, threads):
    """2-layer GCN and 4-layer AGNN on the R-MAT workload.  Every layer is checked on its own: its
    input is the ORACLE's previous-layer output re-rounded to the storage dtype, so errors do not
    compound; the chained GPU result is compared as well and reported."""
    seed = synth.CONFIGS[5]["seed"]
    g = synth.config_graph(5)
    say(f"cfg5 n={g.n} nnz={g.nnz}")
    Xd, X64 = quantise(synth.normal_features(g.n, 128, seed + 10), F16)
    W1d, W1 = quantise(synth.glorot_uniform(128, 16, seed + 11), F16)
    W2d, W2 = quantise(synth.glorot_uniform(16, 8, seed + 12), F16)
    Wind, Win = quantise(synth.glorot_uniform(128, 32, seed + 13), F16)
    Woutd, Wout = quantise(synth.glorot_uniform(32, 8, seed + 14), F16)
    dg = dev_graph(g)
    hp = HotPath(dg)
    hp.build()
    torch.cuda.synchronize()
    check_windows(hp.win, oracle.build_windows(g.row_ptr, g.col_idx))
    say("  window index bit-exact")
    _, dinv64 = oracle.gcn_norm(g.row_ptr, g.col_idx)
    assert np.max(np.abs(hp.dinv.cpu().double().numpy() - dinv64) / dinv64) < 1e-6
    dinv32, fvals64 = factored_vals(g, oracle)
    hp.dinv.copy_(torch.from_numpy(dinv32))          # both sides use the oracle's rounded values

    def f16(x64):
        t = torch.from_numpy(x64).to(F16)
        return t.cuda(), t.double().numpy()

    # ---- GCN
    ref1, ab1 = oracle.gcn_layer(g.row_ptr, g.col_idx, fvals64, X64, W1, relu=True)
    chained = hp.gcn(Xd, W1d, W2d).clone()
    e1 = norm_err(hp.gcn_h, ref1, ab1, F16)
    say(f"  gcn layer 1 err {e1:.3e}")
    assert e1 < 2e-3
    h1d, h1 = f16(ref1)
    ref2, ab2 = oracle.gcn_layer(g.row_ptr, g.col_idx, fvals64, h1, W2)
    out2 = B.ftc_gcn_layer(dg, hp.win, None, h1d, W2d, ws=hp.ws, dinv=hp.dinv)
    e2 = norm_err(out2, ref2, ab2)
    say(f"  gcn layer 2 err {e2:.3e}; chained end-to-end err {norm_err(chained, ref2, ab2):.3e}")
    assert e2 < 2e-3
    del ref1, ab1, ref2, ab2, out2

    # ---- AGNN
    a64, aab = oracle.gemm(X64, Win)
    a64 = np.maximum(a64, 0)
    a_gpu = B.ftc_update_gemm(Xd, Wind, relu=True, out_dtype=F16)
    e = norm_err(a_gpu, a64, aab, F16)
    say(f"  agnn in-projection err {e:.3e}")
    assert e < 2e-3
    chained = hp.agnn(Xd, Wind, Woutd, [1.0] * 4).clone()
    ad, a = f16(a64)
    for layer in range(4):
        ref, ab, _ = oracle.agnn_layer(g.row_ptr, g.col_idx, a, 1.0)
        out = B.ftc_agnn_layer(dg, hp.win, ad, beta=1.0, out_dtype=F16, ws=hp.ws)
        e = norm_err(out, ref, ab, F16)
        say(f"  agnn layer {layer + 1} err {e:.3e}")
        assert e < 2e-3
        ad, a = f16(ref)
    ref, ab = oracle.gemm(a, Wout)
    out = B.ftc_update_gemm(ad, Woutd)
    e = norm_err(out, ref, ab)
    say(f"  agnn out-projection err {e:.3e}; chained end-to-end err {norm_err(chained, ref, ab):.3e}")
    assert e < 2e-3


def test_cfg5_reorder_full():
    """Degree order and relabelled CSR of the R-MAT workload, every entry, against the oracle."""
    from oracle import ftc_oracle_reorder as OR
    g = synth.config_graph(5)
    dg = dev_graph(g)
    for mode in (B.FTC_ORDER_DEGREE, B.FTC_ORDER_DEGREE_CLASSES):
        say(f"cfg5 reorder mode {mode}")
        perm_ref, inv_ref = OR.degree_order(g.row_ptr, mode)
        perm, inv = B.ftc_degree_order(dg, mode)
        assert np.array_equal(perm.cpu().numpy(), perm_ref)
        assert np.array_equal(inv.cpu().numpy(), inv_ref)
        pg, flag = B.ftc_permute_graph(dg, perm, inv)
        assert int(flag.item()) == 0
        rp_ref, ci_ref = OR.permute_graph(g.row_ptr, g.col_idx, perm_ref, inv_ref)
        assert np.array_equal(pg.row_ptr.cpu().numpy(), rp_ref)
        assert np.array_equal(pg.col_idx.cpu().numpy(), ci_ref)
        del pg, rp_ref, ci_ref


def test_cfg5_quarter_backward_every_element(oracle, threads):
    """Backward of a GCN layer and an AGNN layer on the R-MAT recipe at a quarter of the benchmark
    size (262 144 nodes, 8 M entries, hub rows of tens of thousands of entries): every gradient
    element against the numpy backward oracle, which needs minutes and gigabytes beyond that size."""
    from oracle import ftc_oracle_backward as OB
    from test_gpu_backward import term_err
    g = synth.config_graph(5, 0.25)
    say(f"cfg5/4 n={g.n} nnz={g.nnz}")
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    dinv32, fvals64 = factored_vals(g, oracle)
    dinv = torch.from_numpy(dinv32).cuda()
    Xd, X64 = quantise(synth.normal_features(g.n, 32, 5), F16)
    Wd, W64 = quantise(synth.glorot_uniform(32, 16, 6), F16)
    dY32 = synth.normal_features(g.n, 16, 7).astype(np.float32)
    Y = B.ftc_gcn_layer(dg, win, None, Xd, Wd, relu=True, dinv=dinv)
    dX, dW = B.ftc_gcn_layer_backward(dg, win, None, Xd, Wd, torch.from_numpy(dY32).cuda(), Y=Y, dinv=dinv)
    dX_ref, dW_ref, _ = OB.gcn_layer_backward(g.row_ptr, g.col_idx, fvals64, X64, W64, dY32.astype(np.float64),
                                              Y.cpu().double().numpy())
    tX, tW, _ = OB.gcn_layer_backward_terms(g.row_ptr, g.col_idx, fvals64, X64, W64, dY32.astype(np.float64),
                                            Y.cpu().double().numpy())
    ex, ew = term_err(dX, dX_ref, tX), term_err(dW, dW_ref, tW)
    say(f"  gcn backward dX err {ex:.3e} dW err {ew:.3e}")
    assert ex < 1e-5 and ew < 1e-5
    del dX_ref, dX
    Hd, H64 = quantise(synth.normal_features(g.n, 32, 8), F16)
    dYd, dY64 = quantise(synth.normal_features(g.n, 32, 9), F16)
    T, flag = B.ftc_transpose_index(dg, win)
    assert int(flag.item()) == 0
    p = torch.empty(g.nnz, dtype=F32, device="cuda")
    B.ftc_agnn_layer(dg, win, Hd, beta=1.0, edge_p=p)
    dH, dbeta = B.ftc_agnn_layer_backward(dg, win, T, Hd, p, dYd, beta=1.0)
    dH_ref, dbeta_ref = OB.agnn_layer_backward(g.row_ptr, g.col_idx, H64, 1.0, dY64)
    tH, tb = OB.agnn_layer_backward_terms(g.row_ptr, g.col_idx, H64, 1.0, dY64)
    eh, eb = term_err(dH, dH_ref, tH), abs(float(dbeta.item()) - dbeta_ref) / tb
    say(f"  agnn backward dH err {eh:.3e} dbeta {float(dbeta.item()):.6g} ref {dbeta_ref:.6g} err {eb:.3e}")
    assert eh < 1e-5 and eb < 1e-5


def test_cfg5_backward_identities_full():
    """Backward pass at the full benchmark size, in the buffers bench.py --train times (TrainPath),
    checked through identities that hold at any size.  Both models are positively homogeneous of
    degree one in their parameters / inputs (ReLU and the cosine softmax included), so by Euler's
    theorem <dL/dW, W> = <dL/dX, X> = L for the loss L = <dOut, out> of a GCN layer and
    <dL/dH, H> = L for an AGNN layer; dL/dbeta is compared with a central difference of the GPU
    forward pass (itself checked against the oracle at this size above)."""
    from paper_2412_12218_amd.models import TrainPath
    seed = synth.CONFIGS[5]["seed"]
    g = synth.config_graph(5)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    _, dinv = B.ftc_gcn_norm(dg, win, want_vals=False)
    tp = TrainPath(dg, win, dinv)
    dev = dinv.device
    h16 = lambda a: torch.from_numpy(a).to(F16).to(dev)
    X = h16(synth.normal_features(g.n, 128, seed + 10))
    W1, W2 = h16(synth.glorot_uniform(128, 16, seed + 11)), h16(synth.glorot_uniform(16, 8, seed + 12))
    d_out = torch.from_numpy(synth.normal_features(g.n, 8, seed + 21)).to(dev)
    out = tp.gcn_forward(X, W1, W2)
    L = float((out.double() * d_out.double()).sum())
    dW1, dW2 = tp.gcn_backward(X, W1, W2, d_out)
    scale = float((out.double().abs() * d_out.double().abs()).sum())
    l1, l2 = float((dW1.double() * W1.double()).sum()), float((dW2.double() * W2.double()).sum())
    say(f"  gcn: L {L:.6g} <dW1,W1> {l1:.6g} <dW2,W2> {l2:.6g} (sum of |terms| {scale:.3g})")
    # the hidden activations are rounded to fp16 between the layers: 2^-11 relative per element
    assert abs(l1 - L) < 2e-3 * scale and abs(l2 - L) < 2e-3 * scale
    H0 = h16(synth.normal_features(g.n, 32, seed + 20))
    d_agnn = h16(synth.normal_features(g.n, 32, seed + 22))
    betas = [1.0]
    tp1 = TrainPath(dg, win, dinv, agnn_layers=1)
    Y = tp1.agnn_forward(H0, betas)
    L = float((Y.double() * d_agnn.double()).sum())
    scale = float((Y.double().abs() * d_agnn.double().abs()).sum())
    dH, dbeta = tp1.agnn_backward(betas, d_agnn)
    lh = float((dH.double() * H0.double()).sum())
    say(f"  agnn: L {L:.6g} <dH,H> {lh:.6g} (sum of |terms| {scale:.3g})")
    assert abs(lh - L) < 2e-3 * scale
    eps = 1e-2
    Yp = B.ftc_agnn_layer(dg, win, H0, beta=1.0 + eps)
    Ym = B.ftc_agnn_layer(dg, win, H0, beta=1.0 - eps)
    fd = float(((Yp.double() - Ym.double()) * d_agnn.double()).sum()) / (2 * eps)
    say(f"  agnn: dbeta {float(dbeta[0]):.6g} central difference {fd:.6g}")
    assert abs(float(dbeta[0]) - fd) < 2e-2 * max(abs(fd), 1e-3 * scale)


def test_cfg4_label_propagation():
    """Label propagation on the permuted block model: every label against the oracle at a tenth of
    the benchmark size; at the full size (1000 blocks of 1000 nodes) through what the planted
    partition fixes: one label per block, holding nearly all nodes, and a relabelled graph whose
    windows hold fewer distinct columns."""
    from oracle import ftc_oracle_reorder as OR
    g = synth.config_graph(4, 0.1)
    say(f"cfg4/10 n={g.n} nnz={g.nnz}")
    ref = OR.label_propagation(g.row_ptr, g.col_idx, 6)
    lab = B.ftc_label_propagation(dev_graph(g), 6)
    assert np.array_equal(lab.cpu().numpy(), ref)
    g = synth.config_graph(4)
    dg = dev_graph(g)
    lab = B.ftc_label_propagation(dg, 10)
    counts = np.bincount(lab.cpu().numpy(), minlength=g.n)
    big = counts[counts >= 500]
    say(f"cfg4 n={g.n}: {np.count_nonzero(counts)} labels, {big.size} with at least 500 nodes covering {big.sum()} nodes")
    assert big.size == 1000 and big.sum() >= 0.97 * g.n
    perm, inv, flag = B.ftc_order_by_key(lab)
    assert int(flag.item()) == 0
    pn = perm.cpu().numpy()
    assert np.array_equal(np.sort(pn), np.arange(g.n)) and np.array_equal(inv.cpu().numpy()[pn], np.arange(g.n))
    ln = lab.cpu().numpy()[pn]
    assert np.all(np.diff(ln) >= 0)                                   # grouped by label, ...
    same = np.flatnonzero(np.diff(ln) == 0)
    assert np.all(pn[same] < pn[same + 1])                            # ... ascending id inside a label
    pg, pflag = B.ftc_permute_graph(dg, perm, inv)
    assert int(pflag.item()) == 0
    before = int(B.ftc_build_windows(dg).summary[0].item())
    after = int(B.ftc_build_windows(pg).summary[0].item())
    say(f"  distinct window columns {before} -> {after}")
    assert after < 0.9 * before
