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
from paper_2412_12218_amd.models import HotPath

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
