"""GPU parity of the backward pass: every backward entry point of libftc, called through the C
ABI, against the fp64 backward oracle on the same seeded inputs.

Integer outputs (the transposed index) are bit-exact.  A gradient element is compared the way the
forward results are: |gpu - ref| / (sum of the absolute values of the terms it is made of), the
backward oracle's `*_terms` functions giving that sum for every element, and must stay below 1e-5 for
every input type: the oracle gets the rounded 16-bit inputs exactly and every intermediate of the
backward pass is fp32.  A chain of layers is held to the same bar, against terms carried through the
chain."""
import numpy as np
import pytest
import scipy.sparse as sp
import torch

import synth
from oracle import ftc_oracle_backward as OB
from parity import dev_graph, quantise
from paper_2412_12218_amd import binding as B

pytestmark = pytest.mark.gpu

F32, F16, BF16 = torch.float32, torch.float16, torch.bfloat16
GTOL = {F32: 1e-5, F16: 1e-5, BF16: 1e-5}


def say(msg):
    print(msg, flush=True)


def term_err(got, ref, terms):
    """max |got - ref| / terms, elementwise; where no term contributes the result must be exactly zero."""
    got = got.detach().cpu().double().numpy() if torch.is_tensor(got) else np.asarray(got, dtype=np.float64)
    assert np.all(np.isfinite(got))
    terms = np.broadcast_to(terms, ref.shape)
    assert np.all(got[terms == 0] == 0)
    return float(np.max(np.abs(got - ref) / np.where(terms > 0, terms, 1.0))) if ref.size else 0.0


def directed_graph(n, m, seed):
    """Non-symmetric pattern with ascending, duplicate-free rows, a few empty rows, self-loops on
    half the nodes."""
    rng = np.random.default_rng(seed)
    u = np.concatenate([rng.integers(0, n, size=m), np.arange(0, n, 2)])
    v = np.concatenate([rng.integers(0, n, size=m), np.arange(0, n, 2)])
    keep = (u % 97) != 5                               # rows 5, 102, ... stay empty
    A = sp.csr_matrix((np.ones(keep.sum()), (u[keep], v[keep])), shape=(n, n))
    A.sum_duplicates()
    A.sort_indices()
    return synth.Graph(n, A.indptr.astype(np.int32), A.indices.astype(np.int32), "directed")


def host_transpose(g, vals):
    """CSR of the transposed matrix with every stored entry kept (stable order inside a row)."""
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    order = np.argsort(g.col_idx, kind="stable")
    rpT = np.zeros(g.n + 1, dtype=np.int32)
    rpT[1:] = np.cumsum(np.bincount(g.col_idx, minlength=g.n))
    gT = synth.Graph(g.n, rpT, rows[order].astype(np.int32), "T")
    return gT, (None if vals is None else vals[order])


@pytest.fixture(scope="module")
def graphs():
    return {
        "cfg1": synth.config_graph(1),
        "cfg3s": synth.config_graph(3, 0.1),
        "cfg5s": synth.config_graph(5, 1 / 32),
        "directed": directed_graph(5003, 40_000, seed=5),
    }


# ------------------------------------------------------------------ transposed index (bit-exact)
@pytest.mark.parametrize("name", ["cfg1", "cfg3s", "cfg5s", "directed"])
@pytest.mark.parametrize("with_windows", [True, False])
def test_transpose_index(graphs, name, with_windows):
    g = graphs[name]
    say(f"transpose_index {name} n={g.n} nnz={g.nnz} windows={with_windows}")
    ref = OB.transpose_index(g.row_ptr, g.col_idx)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg) if with_windows else None
    T, flag = B.ftc_transpose_index(dg, win)
    assert np.array_equal(T.cpu().numpy().astype(np.int64), ref)
    assert int(flag.item()) == int((ref < 0).any())
    if name == "directed":
        assert (ref < 0).any() and (ref >= 0).any()


def test_transpose_index_empty_graph():
    g = synth.Graph(40, np.zeros(41, dtype=np.int32), np.zeros(0, dtype=np.int32), "empty")
    T, flag = B.ftc_transpose_index(dev_graph(g))
    assert T.numel() == 0 and int(flag.item()) == 0


# ------------------------------------------------------------------ softmax backward
def long_row_graph():
    """Rows of every class of the kernel: empty, a few entries, hundreds, one above 2048."""
    rng = np.random.default_rng(3)
    n = 3000
    deg = rng.integers(0, 14, size=n)
    deg[7] = 0
    deg[100:110] = 300
    deg[555] = 2048
    deg[556] = 2049
    deg[1200] = 9000
    deg[n - 1] = 17
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(deg)
    col = rng.integers(0, n, size=int(row_ptr[-1])).astype(np.int32)
    return synth.Graph(n, row_ptr, col, "long_rows")


@pytest.mark.parametrize("name", ["cfg1", "cfg5s", "long_rows"])
@pytest.mark.parametrize("with_windows", [True, False])
def test_edge_softmax_backward(oracle, graphs, name, with_windows):
    g = long_row_graph() if name == "long_rows" else graphs[name]
    say(f"softmax_backward {name} n={g.n} nnz={g.nnz}")
    rng = np.random.default_rng(8)
    s = rng.normal(size=g.nnz).astype(np.float32) * 3
    p64 = oracle.edge_softmax(g.row_ptr, s.astype(np.float64))
    p32 = p64.astype(np.float32)
    dp32 = rng.normal(size=g.nnz).astype(np.float32)
    ref = OB.edge_softmax_backward(g.row_ptr, p32.astype(np.float64), dp32.astype(np.float64))
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg) if with_windows else None      # entry-balanced kernels / row kernel
    p, dp = torch.from_numpy(p32).cuda(), torch.from_numpy(dp32).cuda()
    ds = B.ftc_edge_softmax_backward(dg, win, p, dp)
    # every term is bounded by p * (|dp| + sum p |dp|): compare against that
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    ab = np.zeros(g.n)
    np.add.at(ab, rows, p32.astype(np.float64) * np.abs(dp32))
    bound = p32.astype(np.float64) * (np.abs(dp32) + ab[rows])
    got = ds.cpu().double().numpy()
    err = float(np.max(np.abs(got - ref) / np.where(bound > 0, bound, 1.0)))
    say(f"  err {err:.3e}")
    assert err < 1e-5
    assert np.all(got[bound == 0] == 0)
    ds2 = B.ftc_edge_softmax_backward(dg, win, p, dp.clone(), out=None)
    assert torch.equal(ds, ds2)
    dpc = dp.clone()
    B.ftc_edge_softmax_backward(dg, win, p, dpc, out=dpc)      # in place
    assert torch.equal(dpc, ds)


# ------------------------------------------------------------------ weight gradient
@pytest.mark.parametrize("n", [1, 15, 1000, 70_001])
@pytest.mark.parametrize("dtype,d_in,d_out", [(F32, 16, 16), (F16, 64, 16), (BF16, 30, 7), (F16, 128, 32),
                                              (F32, 5, 64)])
def test_weight_grad(n, dtype, d_in, d_out):
    say(f"weight_grad n={n} {dtype} {d_in}x{d_out}")
    Xd, X64 = quantise(synth.uniform_features(n, d_in, seed=1), dtype)
    G32 = synth.normal_features(n, d_out, seed=2).astype(np.float32)
    ref = X64.T @ G32.astype(np.float64)
    ab = np.abs(X64).T @ np.abs(G32).astype(np.float64)
    G = torch.from_numpy(G32).cuda()
    dW = B.ftc_weight_grad(Xd, G)
    err = float(np.max(np.abs(dW.cpu().double().numpy() - ref) / ab))
    say(f"  err {err:.3e}")
    assert err < 1e-5
    assert torch.equal(dW, B.ftc_weight_grad(Xd, G))          # fixed summation order


@pytest.mark.parametrize("dtype,d_in,d_out", [(F16, 1432, 16), (F16, 1433, 16), (F32, 3703, 6), (BF16, 520, 64),
                                              (F32, 300, 128), (F16, 40, 300), (F32, 257, 1)])
def test_weight_grad_wide(dtype, d_in, d_out):
    """More input columns than one pass covers: groups of input columns (the last one ragged), and output
    widths that shrink the group."""
    n = 2000 + 3
    say(f"weight_grad wide {dtype} {d_in}x{d_out}")
    Xd, X64 = quantise(synth.uniform_features(n, d_in, seed=1), dtype)
    G32 = synth.normal_features(n, d_out, seed=2).astype(np.float32)
    ref = X64.T @ G32.astype(np.float64)
    ab = np.abs(X64).T @ np.abs(G32).astype(np.float64)
    G = torch.from_numpy(G32).cuda()
    dW = B.ftc_weight_grad(Xd, G)
    assert float(np.max(np.abs(dW.cpu().double().numpy() - ref) / ab)) < 1e-5
    assert torch.equal(dW, B.ftc_weight_grad(Xd, G))


@pytest.mark.parametrize("dtype,d_in,d_out", [(F16, 1432, 16), (F32, 1433, 7), (F16, 128, 128), (BF16, 96, 80),
                                              (F32, 70, 130), (F16, 264, 256)])
def test_update_gemm_backward_wide_input(dtype, d_in, d_out):
    """The first layer of a model on a wide feature matrix, and hidden sizes above 64 (the input gradient
    then runs as a dense update with the transposed weights): forward, then dW and dX."""
    n = 1500 + 1
    Xd, X64 = quantise(synth.uniform_features(n, d_in, seed=1), dtype)
    Wd, W64 = quantise(synth.glorot_uniform(d_in, d_out, seed=2), dtype)
    dZ32 = synth.normal_features(n, d_out, seed=3).astype(np.float32)
    Z = B.ftc_update_gemm(Xd, Wd, relu=True, out_dtype=dtype)
    dX_ref, dW_ref = OB.update_gemm_backward(X64, W64, dZ32.astype(np.float64), Z.cpu().double().numpy())
    tX, tW = OB.update_gemm_backward_terms(X64, W64, dZ32.astype(np.float64), Z.cpu().double().numpy())
    dX, dW = B.ftc_update_gemm_backward(Xd, Wd, torch.from_numpy(dZ32).cuda(), Z=Z)
    ex, ew = term_err(dX, dX_ref, tX), term_err(dW, dW_ref, tW)
    say(f"update_gemm_backward wide {dtype} {d_in}->{d_out}: dX err {ex:.3e} dW err {ew:.3e}")
    assert ex < 1e-5 and ew < 1e-5


@pytest.mark.parametrize("dtype,d_in,d_out", [(F16, 64, 128), (F32, 40, 72)])
def test_gcn_layer_backward_wide_hidden(oracle, graphs, dtype, d_in, d_out):
    g = graphs["cfg1"]
    vals64, _ = oracle.gcn_norm(g.row_ptr, g.col_idx)
    vals32 = vals64.astype(np.float32)
    Xd, X64 = quantise(synth.uniform_features(g.n, d_in, seed=4), dtype)
    Wd, W64 = quantise(synth.glorot_uniform(d_in, d_out, seed=5), dtype)
    dY32 = synth.normal_features(g.n, d_out, seed=6).astype(np.float32)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    vd = torch.from_numpy(vals32).cuda()
    Y = B.ftc_gcn_layer(dg, win, vd, Xd, Wd, relu=True)
    dX_ref, dW_ref, _ = OB.gcn_layer_backward(g.row_ptr, g.col_idx, vals32.astype(np.float64), X64, W64,
                                              dY32.astype(np.float64), Y.cpu().double().numpy())
    tX, tW, _ = OB.gcn_layer_backward_terms(g.row_ptr, g.col_idx, vals32.astype(np.float64), X64, W64,
                                            dY32.astype(np.float64), Y.cpu().double().numpy())
    dX, dW = B.ftc_gcn_layer_backward(dg, win, vd, Xd, Wd, torch.from_numpy(dY32).cuda(), Y=Y)
    ex, ew = term_err(dX, dX_ref, tX), term_err(dW, dW_ref, tW)
    say(f"gcn_layer_backward wide hidden {dtype}: dX err {ex:.3e} dW err {ew:.3e}")
    assert ex < 1e-5 and ew < 1e-5


def test_weight_grad_strided_inputs():
    n, d_in, d_out = 777, 20, 12
    Xf = torch.from_numpy(synth.uniform_features(n, 40, seed=3)).to(F16).cuda()
    Gf = torch.from_numpy(synth.normal_features(n, 16, seed=4).astype(np.float32)).cuda()
    X, G = Xf[:, :d_in], Gf[:, :d_out]
    ref = X.double().cpu().numpy().T @ G.double().cpu().numpy()
    ab = X.double().abs().cpu().numpy().T @ G.double().abs().cpu().numpy()
    dW = B.ftc_weight_grad(X, G)
    assert term_err(dW, ref, ab) < 1e-5


# ------------------------------------------------------------------ dense update backward
@pytest.mark.parametrize("n", [1, 1000, 70_001])
@pytest.mark.parametrize("dtype,d_in,d_out", [(F16, 128, 32), (F32, 16, 16), (BF16, 30, 7), (F16, 32, 8)])
@pytest.mark.parametrize("relu", [False, True])
def test_update_gemm_backward(n, dtype, d_in, d_out, relu):
    say(f"update_gemm_backward n={n} {dtype} {d_in}->{d_out} relu={relu}")
    Xd, X64 = quantise(synth.uniform_features(n, d_in, seed=1), dtype)
    Wd, W64 = quantise(synth.glorot_uniform(d_in, d_out, seed=2), dtype)
    dZ32 = synth.normal_features(n, d_out, seed=3).astype(np.float32)
    Z = B.ftc_update_gemm(Xd, Wd, relu=True, out_dtype=dtype) if relu else None      # the mask is the layer's own output
    dX_ref, dW_ref = OB.update_gemm_backward(X64, W64, dZ32.astype(np.float64), Z.cpu().double().numpy() if relu else None)
    tX, tW = OB.update_gemm_backward_terms(X64, W64, dZ32.astype(np.float64), Z.cpu().double().numpy() if relu else None)
    dZ = torch.from_numpy(dZ32).cuda()
    dX, dW = B.ftc_update_gemm_backward(Xd, Wd, dZ, Z=Z)
    ex, ew = term_err(dX, dX_ref, tX), term_err(dW, dW_ref, tW)
    say(f"  dX err {ex:.3e} dW err {ew:.3e}")
    assert ex < 1e-5 and ew < 1e-5
    dX16, dW2 = B.ftc_update_gemm_backward(Xd, Wd, dZ, Z=Z, dx_dtype=F16)
    assert torch.equal(dX16, dX.to(F16)) and torch.equal(dW2, dW)
    none, dW3 = B.ftc_update_gemm_backward(Xd, Wd, dZ, Z=Z, want_dX=False)
    assert none is None and torch.equal(dW3, dW)


# ------------------------------------------------------------------ GCN layer backward
@pytest.mark.parametrize("name", ["cfg1", "cfg3s", "cfg5s", "directed"])
@pytest.mark.parametrize("dtype,d_in,d_out", [(F16, 64, 16), (F32, 16, 16), (BF16, 30, 7), (F16, 16, 40)])
@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("factored", [False, True])
def test_gcn_layer_backward(oracle, graphs, name, dtype, d_in, d_out, relu, factored):
    g = graphs[name]
    if name in ("cfg3s", "cfg5s") and (dtype, d_in, d_out) not in ((F16, 64, 16), (F32, 16, 16)):
        pytest.skip("odd shapes are covered on the small graphs")
    say(f"gcn_layer_backward {name} {dtype} {d_in}->{d_out} relu={relu} factored={factored}")
    _, dinv64 = oracle.gcn_norm(g.row_ptr, g.col_idx)
    dinv32 = np.nan_to_num(dinv64, posinf=0.0).astype(np.float32)       # empty rows: 0
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    vals_ref = dinv32[rows].astype(np.float64) * dinv32[g.col_idx].astype(np.float64)
    if factored:
        vals32 = None
    else:
        vals32 = vals_ref.astype(np.float32)
        vals_ref = vals32.astype(np.float64)
    Xd, X64 = quantise(synth.uniform_features(g.n, d_in, seed=9), dtype)
    Wd, W64 = quantise(synth.glorot_uniform(d_in, d_out, seed=10), dtype)
    dY32 = synth.normal_features(g.n, d_out, seed=13).astype(np.float32)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    dinv_d = torch.from_numpy(dinv32).cuda() if factored else None
    vals_d = torch.from_numpy(vals32).cuda() if vals32 is not None else None
    # forward on the GPU: the ReLU mask of the backward pass is the layer's own output
    Y = B.ftc_gcn_layer(dg, win, vals_d, Xd, Wd, relu=relu, dinv=dinv_d) if relu else None
    Y64 = Y.cpu().double().numpy() if relu else None
    dX_ref, dW_ref, _ = OB.gcn_layer_backward(g.row_ptr, g.col_idx, vals_ref, X64, W64,
                                              dY32.astype(np.float64), Y64)
    # the transposed operator: the graph itself when the pattern is symmetric
    if name == "directed":
        gT, valsT = host_transpose(g, vals32)
        dgT = dev_graph(gT)
        winT = B.ftc_build_windows(dgT)
        valsT_d = torch.from_numpy(valsT).cuda() if valsT is not None else None
    else:
        dgT, winT, valsT_d = dg, win, vals_d
    dY = torch.from_numpy(dY32).cuda()
    tX, tW, _ = OB.gcn_layer_backward_terms(g.row_ptr, g.col_idx, vals_ref, X64, W64, dY32.astype(np.float64), Y64)
    dX, dW = B.ftc_gcn_layer_backward(dgT, winT, valsT_d, Xd, Wd, dY, Y=Y, dinv=dinv_d)
    ex, ew = term_err(dX, dX_ref, tX), term_err(dW, dW_ref, tW)
    say(f"  dX err {ex:.3e} dW err {ew:.3e}")
    assert ex < GTOL[dtype] and ew < GTOL[dtype]
    dX2, dW2 = B.ftc_gcn_layer_backward(dgT, None, valsT_d, Xd, Wd, dY, Y=Y, dinv=dinv_d)   # row kernels
    assert term_err(dX2, dX_ref, tX) < GTOL[dtype] and term_err(dW2, dW_ref, tW) < GTOL[dtype]
    none, dW3 = B.ftc_gcn_layer_backward(dgT, winT, valsT_d, Xd, Wd, dY, Y=Y, dinv=dinv_d, want_dX=False)
    assert none is None and torch.equal(dW3, dW)


# ------------------------------------------------------------------ AGNN layer backward
@pytest.mark.parametrize("name", ["cfg1", "cfg3s", "cfg5s"])
@pytest.mark.parametrize("dtype,D", [(F32, 16), (F16, 32), (BF16, 24), (F16, 64), (F32, 5)])
@pytest.mark.parametrize("beta", [1.0, -2.5])
def test_agnn_layer_backward(graphs, name, dtype, D, beta):
    g = graphs[name]
    if name != "cfg1" and (dtype, D) not in ((F32, 16), (F16, 32)):
        pytest.skip("odd widths are covered on the small graph")
    say(f"agnn_layer_backward {name} {dtype} D={D} beta={beta}")
    Hd, H64 = quantise(synth.normal_features(g.n, D, seed=11), dtype)
    dYd, dY64 = quantise(synth.normal_features(g.n, D, seed=14), dtype)
    dH_ref, dbeta_ref = OB.agnn_layer_backward(g.row_ptr, g.col_idx, H64, beta, dY64)
    tH, tb = OB.agnn_layer_backward_terms(g.row_ptr, g.col_idx, H64, beta, dY64)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    T, flag = B.ftc_transpose_index(dg, win)
    assert int(flag.item()) == 0
    p = torch.empty(g.nnz, dtype=F32, device="cuda")
    B.ftc_agnn_layer(dg, win, Hd, beta=beta, edge_p=p)       # forward pass keeps its probabilities
    dH, dbeta = B.ftc_agnn_layer_backward(dg, win, T, Hd, p, dYd, beta=beta)
    eh = term_err(dH, dH_ref, tH)
    db = abs(float(dbeta.item()) - dbeta_ref) / tb
    say(f"  dH err {eh:.3e} dbeta {float(dbeta.item()):.6g} ref {dbeta_ref:.6g} err {db:.2e}")
    assert eh < GTOL[dtype]
    assert db < 1e-5
    dH2, dbeta2 = B.ftc_agnn_layer_backward(dg, None, T, Hd, p, dYd, beta=beta)      # row kernels
    assert term_err(dH2, dH_ref, tH) < GTOL[dtype]
    assert abs(float(dbeta2.item()) - dbeta_ref) / tb < 1e-5
    dH3, dbeta3 = B.ftc_agnn_layer_backward(dg, win, T, Hd, p, dYd, beta=beta)
    assert torch.equal(dH, dH3) and torch.equal(dbeta, dbeta3)


# ------------------------------------------------------------------ single-pass AGNN backward
@pytest.mark.parametrize("name", ["cfg1", "cfg3s", "cfg5s"])
@pytest.mark.parametrize("dtype,D", [(F32, 16), (F16, 32), (BF16, 24), (F16, 64), (F32, 12), (F16, 8), (F16, 128),
                                     (F32, 64)])
@pytest.mark.parametrize("beta", [1.0, -2.5])
def test_agnn_forward_row_z_and_fused_backward(oracle, graphs, name, dtype, D, beta):
    g = graphs[name]
    if name != "cfg1" and (dtype, D) not in ((F32, 16), (F16, 32)):
        pytest.skip("odd widths are covered on the small graph")
    say(f"agnn fused backward {name} {dtype} D={D} beta={beta}")
    Hd, H64 = quantise(synth.normal_features(g.n, D, seed=11), dtype)
    dYd, dY64 = quantise(synth.normal_features(g.n, D, seed=14), dtype)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    row_z = torch.empty(g.n, dtype=F32, device="cuda")
    Y = B.ftc_agnn_layer(dg, win, Hd, beta=beta, row_z=row_z)           # fp32 output of the single-pass forward
    z_ref = OB.agnn_row_z(g.row_ptr, g.col_idx, H64, beta)
    ez = float(np.max(np.abs(row_z.cpu().double().numpy() - z_ref) / np.maximum(z_ref, 1e-300)))
    say(f"  row_z err {ez:.3e}")
    assert ez < 1e-5
    assert torch.equal(Y, B.ftc_agnn_layer(dg, win, Hd, beta=beta))    # the extra output changes nothing
    dH_ref, dbeta_ref = OB.agnn_layer_backward(g.row_ptr, g.col_idx, H64, beta, dY64)
    tH, tb = OB.agnn_layer_backward_terms(g.row_ptr, g.col_idx, H64, beta, dY64)
    dH, dbeta = B.ftc_agnn_layer_backward_fused(dg, win, Hd, row_z, Y, dYd, beta=beta)
    eh = term_err(dH, dH_ref, tH)
    db = abs(float(dbeta.item()) - dbeta_ref) / tb
    say(f"  dH err {eh:.3e} dbeta {float(dbeta.item()):.6g} ref {dbeta_ref:.6g} err {db:.2e}")
    assert eh < GTOL[dtype]                                             # fp32 Y: the full-precision bar
    assert db < 1e-5
    dH2, dbeta2 = B.ftc_agnn_layer_backward_fused(dg, win, Hd, row_z, Y, dYd, beta=beta)
    assert torch.equal(dH, dH2) and torch.equal(dbeta, dbeta2)
    if dtype != F32:
        # the layer's output in the activation type plus its unrounded copy: what a 16-bit layer stack keeps
        y32 = torch.empty((g.n, (D + 3) // 4 * 4), dtype=F32, device="cuda")
        Y16 = B.ftc_agnn_layer(dg, win, Hd, beta=beta, out_dtype=dtype, row_z=row_z, out_f32=y32)
        assert torch.equal(y32[:, :D], Y) and torch.equal(Y16, Y.to(dtype))
        dH16, dbeta16 = B.ftc_agnn_layer_backward_fused(dg, win, Hd, row_z, y32[:, :D], dYd, beta=beta, dh_dtype=dtype)
        assert torch.equal(dH16, dH.to(dtype)) and torch.equal(dbeta16, dbeta)


def test_agnn_fused_backward_matches_the_unfused_route_on_hub_rows():
    """Rows far longer than a wave's range (thousands of entries) and empty rows: both routes of the
    backward pass against each other and against the oracle."""
    rng = np.random.default_rng(12)
    n = 6000
    import scipy.sparse as sp
    u = np.concatenate([rng.integers(0, n, size=20_000), np.full(4000, 77), np.full(1500, 3001)])
    v = np.concatenate([rng.integers(0, n, size=20_000), rng.integers(0, n, size=4000), rng.integers(0, n, size=1500)])
    keep = (u % 50 != 9) & (v % 50 != 9)                      # nodes 9, 59, ... stay isolated: empty rows
    A = sp.csr_matrix((np.ones(keep.sum()), (u[keep], v[keep])), shape=(n, n))
    A = (A + A.T).tocsr()
    A.sum_duplicates()
    A.sort_indices()
    g = synth.Graph(n, A.indptr.astype(np.int32), A.indices.astype(np.int32), "hubs")
    assert np.diff(g.row_ptr).max() > 2000 and np.diff(g.row_ptr).min() == 0
    Hd, H64 = quantise(synth.normal_features(n, 32, seed=1), F16)
    dYd, dY64 = quantise(synth.normal_features(n, 32, seed=2), F16)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    T, flag = B.ftc_transpose_index(dg, win)
    assert int(flag.item()) == 0
    p = torch.empty(g.nnz, dtype=F32, device="cuda")
    B.ftc_agnn_layer(dg, win, Hd, beta=2.0, edge_p=p)
    dH_u, db_u = B.ftc_agnn_layer_backward(dg, win, T, Hd, p, dYd, beta=2.0)
    row_z = torch.empty(n, dtype=F32, device="cuda")
    Y = B.ftc_agnn_layer(dg, win, Hd, beta=2.0, row_z=row_z)
    dH_f, db_f = B.ftc_agnn_layer_backward_fused(dg, win, Hd, row_z, Y, dYd, beta=2.0)
    dH_ref, db_ref = OB.agnn_layer_backward(g.row_ptr, g.col_idx, H64, 2.0, dY64)
    tH, tb = OB.agnn_layer_backward_terms(g.row_ptr, g.col_idx, H64, 2.0, dY64)
    eu, ef = term_err(dH_u, dH_ref, tH), term_err(dH_f, dH_ref, tH)
    say(f"hub rows: unfused err {eu:.3e} fused err {ef:.3e} dbeta {float(db_u.item()):.6g} {float(db_f.item()):.6g} ref {db_ref:.6g}")
    assert eu < 1e-5 and ef < 1e-5
    assert abs(float(db_f.item()) - db_ref) / tb < 1e-5 and abs(float(db_u.item()) - db_ref) / tb < 1e-5
    empty = torch.from_numpy(np.diff(g.row_ptr) == 0).cuda()
    assert torch.all(dH_f[empty] == 0) and torch.all(row_z[empty] == 0)


def test_single_pass_backward_reports_a_pattern_that_is_not_symmetric(graphs):
    """The single-pass route holds on a symmetric pattern only.  Given the flag of ftc_transpose_index it turns
    the gradients of a non-symmetric graph into NaN; on a symmetric graph the flag changes nothing."""
    for name in ("directed", "cfg1"):
        g = graphs[name]
        dg = dev_graph(g)
        win = B.ftc_build_windows(dg)
        _, flag = B.ftc_transpose_index(dg, win)
        Hd, _ = quantise(synth.normal_features(g.n, 32, seed=1), F16)
        dYd, _ = quantise(synth.normal_features(g.n, 32, seed=2), F16)
        row_z = torch.empty(g.n, dtype=F32, device="cuda")
        Y = B.ftc_agnn_layer(dg, win, Hd, beta=1.0, row_z=row_z)
        dH, dbeta = B.ftc_agnn_layer_backward_fused(dg, win, Hd, row_z, Y, dYd, pattern_flag=flag)
        dH16, _ = B.ftc_agnn_layer_backward_fused(dg, win, Hd, row_z, Y, dYd, pattern_flag=flag, dh_dtype=F16)
        if name == "directed":
            assert int(flag.item()) == 1
            assert bool(torch.isnan(dH).all()) and bool(torch.isnan(dbeta).all()) and bool(torch.isnan(dH16).all())
        else:
            assert int(flag.item()) == 0
            dH0, dbeta0 = B.ftc_agnn_layer_backward_fused(dg, win, Hd, row_z, Y, dYd)
            assert torch.equal(dH, dH0) and torch.equal(dbeta, dbeta0) and bool(torch.isfinite(dH).all())


def test_backward_on_a_graph_without_entries():
    g = synth.Graph(70, np.zeros(71, dtype=np.int32), np.zeros(0, dtype=np.int32), "no_edges")
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    H = torch.from_numpy(synth.normal_features(70, 16, seed=1)).to(F16).cuda()
    dY = torch.from_numpy(synth.normal_features(70, 16, seed=2)).to(F16).cuda()
    z = torch.full((70,), -1.0, dtype=F32, device="cuda")
    Y = B.ftc_agnn_layer(dg, win, H, row_z=z)
    assert torch.all(Y == 0) and torch.all(z == 0)
    dH, dbeta = B.ftc_agnn_layer_backward_fused(dg, win, H, z, Y, dY)
    assert torch.all(dH == 0) and float(dbeta.item()) == 0.0
    T, flag = B.ftc_transpose_index(dg, win)
    p = torch.empty(0, dtype=F32, device="cuda")
    dH2, dbeta2 = B.ftc_agnn_layer_backward(dg, win, T, H, p, dY)
    assert torch.all(dH2 == 0) and float(dbeta2.item()) == 0.0
    W = torch.from_numpy(synth.glorot_uniform(16, 8, seed=3)).to(F16).cuda()
    dX, dW = B.ftc_gcn_layer_backward(dg, win, None, H, W, torch.ones((70, 8), dtype=F32, device="cuda"))
    assert torch.all(dX == 0) and torch.all(dW == 0)


def test_agnn_row_z_needs_the_single_pass_route(graphs):
    g = graphs["cfg1"]
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    H = torch.zeros((g.n, 16), dtype=F16, device="cuda")
    z = torch.empty(g.n, dtype=F32, device="cuda")
    with pytest.raises(B.FtcError):
        B.ftc_agnn_layer(dg, None, H, row_z=z)                                    # no window index
    with pytest.raises(B.FtcError):
        B.ftc_agnn_layer(dg, win, H, row_z=z, edge_p=torch.empty(g.nnz, dtype=F32, device="cuda"))
    with pytest.raises(B.FtcError):                                               # 2 * 256 slots: too wide
        B.ftc_agnn_layer_backward_fused(dg, win, torch.zeros((g.n, 256), dtype=F16, device="cuda"), z,
                                        torch.zeros((g.n, 256), dtype=F32, device="cuda"),
                                        torch.zeros((g.n, 256), dtype=F16, device="cuda"))


def test_agnn_layer_backward_zero_rows_and_isolated_nodes():
    """Nodes whose only neighbour is themselves, and an all-zero feature row (its direction is
    undefined: the forward definition clamps the norm, the gradient through it stays finite)."""
    g = synth.config_graph(1)
    D = 16
    H32 = synth.normal_features(g.n, D, seed=21)
    H32[17] = 0.0
    Hd, H64 = quantise(H32, F32)
    dYd, dY64 = quantise(synth.normal_features(g.n, D, seed=22), F32)
    dH_ref, dbeta_ref = OB.agnn_layer_backward(g.row_ptr, g.col_idx, H64, 1.5, dY64)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    T, _ = B.ftc_transpose_index(dg, win)
    p = torch.empty(g.nnz, dtype=F32, device="cuda")
    B.ftc_agnn_layer(dg, win, Hd, beta=1.5, edge_p=p)
    dH, dbeta = B.ftc_agnn_layer_backward(dg, win, T, Hd, p, dYd, beta=1.5)
    tH, tb = OB.agnn_layer_backward_terms(g.row_ptr, g.col_idx, H64, 1.5, dY64)
    # d/dh of h / max(|h|, eps) at h = 0 is 1 / eps: the clamped row is the plain scaling by 1e12 that the
    # forward pass applies (no projection term); its gradient is huge and held to the same relative bar
    assert np.abs(dH_ref[17]).max() > 1e9
    e1 = term_err(dH, dH_ref, tH)
    assert e1 < 1e-5
    assert abs(float(dbeta.item()) - dbeta_ref) / tb < 1e-5
    # the same through the single-pass route
    row_z = torch.empty(g.n, dtype=F32, device="cuda")
    Y = B.ftc_agnn_layer(dg, win, Hd, beta=1.5, row_z=row_z)
    dH2, dbeta2 = B.ftc_agnn_layer_backward_fused(dg, win, Hd, row_z, Y, dYd, beta=1.5)
    e2 = term_err(dH2, dH_ref, tH)
    say(f"zero row and isolated nodes: edge-array route {e1:.3e}, single pass {e2:.3e}")
    assert e2 < 1e-5
    assert abs(float(dbeta2.item()) - dbeta_ref) / tb < 1e-5


def test_agnn_layer_backward_16bit_gradient_output(graphs):
    """dH written in the activation type (what the layer below takes as its incoming gradient):
    the fp32 result rounded once."""
    g = graphs["cfg1"]
    Hd, _ = quantise(synth.normal_features(g.n, 32, seed=11), F16)
    dYd, _ = quantise(synth.normal_features(g.n, 32, seed=14), F16)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    T, _ = B.ftc_transpose_index(dg, win)
    p = torch.empty(g.nnz, dtype=F32, device="cuda")
    B.ftc_agnn_layer(dg, win, Hd, beta=1.0, edge_p=p)
    dH32, db32 = B.ftc_agnn_layer_backward(dg, win, T, Hd, p, dYd)
    for dt in (F16, BF16):
        dH16, db16 = B.ftc_agnn_layer_backward(dg, win, T, Hd, p, dYd, dh_dtype=dt)
        assert dH16.dtype == dt and torch.equal(dH16, dH32.to(dt)) and torch.equal(db16, db32)


@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("sizes", [(24, 16, 12, 8), (300, 128, 40, 10)])
def test_train_path_stacks_against_chained_oracle(oracle, fused, sizes):
    """TrainPath (2-layer GCN, 3 AGNN propagation layers, fp32 activations) against the per-layer
    oracles chained on the CPU; the AGNN layers through the single-pass pair and through the
    edge-array route.  Once with the small widths, once with a 300-column input and a hidden size of 128."""
    from paper_2412_12218_amd.models import TrainPath
    d_feat, hid, dh, n_out = sizes
    g = synth.config_graph(1)
    n = g.n
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    _, dinv = B.ftc_gcn_norm(dg, win)
    tp = TrainPath(dg, win, dinv, d_feat=d_feat, gcn_hidden=hid, agnn_hidden=dh, n_out=n_out, agnn_layers=3, act_dtype=F32,
                   fused=fused)
    assert tp.fused == fused
    dinv64 = dinv.cpu().double().numpy()
    rows = np.repeat(np.arange(n), np.diff(g.row_ptr))
    vals = dinv64[rows] * dinv64[g.col_idx]
    # GCN
    Xd, X64 = quantise(synth.uniform_features(n, d_feat, seed=31), F32)
    W1d, W164 = quantise(synth.glorot_uniform(d_feat, hid, seed=32), F32)
    W2d, W264 = quantise(synth.glorot_uniform(hid, n_out, seed=33), F32)
    dOutd, dOut64 = quantise(synth.normal_features(n, n_out, seed=34), F32)
    tp.gcn_forward(Xd, W1d, W2d)
    dW1, dW2 = tp.gcn_backward(Xd, W1d, W2d, dOutd)
    H1 = tp.gcn_h.cpu().double().numpy()
    dH1_ref, dW2_ref, _ = OB.gcn_layer_backward(g.row_ptr, g.col_idx, vals, H1, W264, dOut64)
    _, dW1_ref, _ = OB.gcn_layer_backward(g.row_ptr, g.col_idx, vals, X64, W164, dH1_ref, Y=H1)
    tH1, tW2, _ = OB.gcn_layer_backward_terms(g.row_ptr, g.col_idx, vals, H1, W264, dOut64)
    _, tW1, _ = OB.gcn_layer_backward_terms(g.row_ptr, g.col_idx, vals, X64, W164, dH1_ref, Y=H1, dY_terms=tH1)
    e1, e2 = term_err(dW1, dW1_ref, tW1), term_err(dW2, dW2_ref, tW2)
    say(f"gcn stack dW1 err {e1:.3e} dW2 err {e2:.3e}")
    assert e1 < 1e-5 and e2 < 1e-5
    # AGNN
    betas = [1.0, -0.7, 2.0]
    H0d, H064 = quantise(synth.normal_features(n, dh, seed=35), F32)
    dYd, dY64 = quantise(synth.normal_features(n, dh, seed=36), F32)
    tp.agnn_forward(H0d, betas)
    dH0, dbeta = tp.agnn_backward(betas, dYd)
    Hs = [H064]
    for l in range(3):
        Hs.append(oracle.agnn_layer(g.row_ptr, g.col_idx, Hs[l], betas[l])[0])
    d, t, db_ref, tb = dY64, None, [0.0] * 3, [0.0] * 3
    for l in reversed(range(3)):
        t, tb[l] = OB.agnn_layer_backward_terms(g.row_ptr, g.col_idx, Hs[l], betas[l], d, dY_terms=t)
        d, db_ref[l] = OB.agnn_layer_backward(g.row_ptr, g.col_idx, Hs[l], betas[l], d)
    eh = term_err(dH0, d, t)
    eb = [abs(float(dbeta[l].item()) - db_ref[l]) / tb[l] for l in range(3)]
    say(f"agnn stack dH0 err {eh:.3e} dbeta {dbeta.cpu().numpy()} ref {db_ref} err {eb}")
    assert eh < 1e-5 and all(e < 1e-5 for e in eb)


@pytest.mark.parametrize("act", [F32, F16])
def test_train_path_whole_agnn_model_against_chained_oracle(oracle, act):
    """In-projection with ReLU, three propagation layers, out-projection: weight and beta gradients of
    TrainPath against the per-layer oracles chained on the CPU.  With fp16 activations the oracle
    chain starts every layer from the GPU's own (rounded) activations, as the layer tests do."""
    from paper_2412_12218_amd.models import TrainPath
    g = synth.config_graph(1)
    n = g.n
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    _, dinv = B.ftc_gcn_norm(dg, win)
    tp = TrainPath(dg, win, dinv, d_feat=24, gcn_hidden=16, agnn_hidden=16, n_out=8, agnn_layers=3, act_dtype=act)
    Xd, X64 = quantise(synth.uniform_features(n, 24, seed=41), act)
    Wid, Wi64 = quantise(synth.glorot_uniform(24, 16, seed=42), act)
    Wod, Wo64 = quantise(synth.glorot_uniform(16, 8, seed=43), act)
    dOutd, dOut64 = quantise(synth.normal_features(n, 8, seed=44), F32)
    betas = [1.0, -0.7, 2.0]
    tp.agnn_model_forward(Xd, Wid, Wod, betas)
    dW_in, dW_out, dbeta = tp.agnn_model_backward(Xd, Wid, Wod, betas, dOutd)
    Hs = [tp.agnn_h0.cpu().double().numpy()] + [tp.agnn_h[l].cpu().double().numpy() for l in (1, 2, 3)]
    d, dWo_ref = OB.update_gemm_backward(Hs[3], Wo64, dOut64)
    t, tWo = OB.update_gemm_backward_terms(Hs[3], Wo64, dOut64)
    db_ref, tb = [0.0] * 3, [0.0] * 3
    for l in reversed(range(3)):
        d_in = torch.from_numpy(d).to(act).double().numpy()      # the chain hands gradients on in the activation type
        t, tb[l] = OB.agnn_layer_backward_terms(g.row_ptr, g.col_idx, Hs[l], betas[l], d_in, dY_terms=t)
        d, db_ref[l] = OB.agnn_layer_backward(g.row_ptr, g.col_idx, Hs[l], betas[l], d_in)
    _, dWi_ref = OB.update_gemm_backward(X64, Wi64, d, Hs[0])
    _, tWi = OB.update_gemm_backward_terms(X64, Wi64, d, Hs[0], dZ_terms=t)
    ei, eo = term_err(dW_in, dWi_ref, tWi), term_err(dW_out, dWo_ref, tWo)
    eb = [abs(float(dbeta[l].item()) - db_ref[l]) / tb[l] for l in range(3)]
    say(f"agnn model ({act}): dW_in err {ei:.3e} dW_out err {eo:.3e} dbeta {dbeta.cpu().numpy()} ref {db_ref} err {eb}")
    # fp16 activations: the gradients handed from layer to layer are rounded to fp16 on both sides, and a value
    # that sits on a rounding boundary may fall either way: the 16-bit bar
    tol = 1e-5 if act == F32 else 2e-3
    assert ei < tol and eo < 1e-5
    assert all(e < tol for e in eb)


def test_train_path_rejects_a_non_symmetric_pattern():
    from paper_2412_12218_amd.models import TrainPath
    g = directed_graph(300, 1500, seed=2)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    _, dinv = B.ftc_gcn_norm(dg, win)
    with pytest.raises(ValueError):
        TrainPath(dg, win, dinv)


def test_backward_rejects_bad_arguments():
    g = synth.config_graph(1)
    dg = dev_graph(g)
    H = torch.zeros((g.n, 16), dtype=F16, device="cuda")
    dY32 = torch.zeros((g.n, 16), dtype=F32, device="cuda")
    T = torch.zeros(g.nnz, dtype=torch.int32, device="cuda")
    p = torch.zeros(g.nnz, dtype=F32, device="cuda")
    with pytest.raises(B.FtcError):        # workspace too small
        B.ftc_agnn_layer_backward(dg, None, T, H, p, H.clone(), ws=torch.empty(256, dtype=torch.uint8, device="cuda"))
    W = torch.zeros((16, 508), dtype=F16, device="cuda")
    with pytest.raises(B.FtcError):        # more output columns than the weight gradient covers
        B.ftc_gcn_layer_backward(dg, None, None, H, W, torch.zeros((g.n, 508), dtype=F32, device="cuda"))
    with pytest.raises(B.FtcError):        # more output columns than a pass of the weight gradient covers
        B.ftc_weight_grad(torch.zeros((10, 16), dtype=F16, device="cuda"),
                          torch.zeros((10, 508), dtype=F32, device="cuda"))
    del dY32


# ------------------------------------------------------------------ seeded sweep over shapes
@pytest.mark.parametrize("case", list(range(16)) + [33, 39, 132, 384])
def test_agnn_backward_random_shapes(case):
    """Symmetric random graphs from 1 to a few thousand nodes (isolated nodes, self-loops on some,
    a long row in the larger ones), widths from 1 to 64: the edge-array route always, the single-pass
    route where it covers the shape, both against the oracle.  (Cases 39 and 132: one-element rows with
    norms down to 1e-4, where the gradient through the direction is exactly zero; case 33: a row with a
    single neighbour on the single-pass route; case 384: a signed sum of one-element rows that nearly cancels.)"""
    import scipy.sparse as sp
    rng = np.random.default_rng(2000 + case)
    n = int(rng.choice([1, 2, 17, 64, 500, 1025, 3000]))
    m = int(n * rng.integers(1, 8))
    u, v = rng.integers(0, n, size=m), rng.integers(0, n, size=m)
    if n >= 500:
        hub = int(rng.integers(0, n))
        u = np.concatenate([u, np.full(900, hub)])
        v = np.concatenate([v, rng.integers(0, n, size=900)])
    loops = np.flatnonzero(rng.random(n) < 0.5)
    A = sp.csr_matrix((np.ones(u.size + loops.size), (np.concatenate([u, loops]), np.concatenate([v, loops]))), shape=(n, n))
    A = (A + A.T).tocsr()
    A.sum_duplicates()
    A.sort_indices()
    g = synth.Graph(n, A.indptr.astype(np.int32), A.indices.astype(np.int32), "random")
    dtype = [F32, F16, BF16][case % 3]
    D = int(rng.choice([1, 3, 4, 8, 12, 16, 24, 32, 40, 64]))
    beta = float(rng.choice([1.0, -1.5, 3.0]))
    say(f"random case {case}: n={n} nnz={g.nnz} {dtype} D={D} beta={beta}")
    Hd, H64 = quantise(synth.normal_features(n, D, seed=case), dtype)
    dYd, dY64 = quantise(synth.normal_features(n, D, seed=100 + case), dtype)
    dH_ref, dbeta_ref = OB.agnn_layer_backward(g.row_ptr, g.col_idx, H64, beta, dY64)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    T, flag = B.ftc_transpose_index(dg, win)
    assert int(flag.item()) == 0
    p = torch.empty(g.nnz, dtype=F32, device="cuda")
    B.ftc_agnn_layer(dg, win, Hd, beta=beta, edge_p=p)
    dH, dbeta = B.ftc_agnn_layer_backward(dg, win, T, Hd, p, dYd, beta=beta)
    tH, tb = OB.agnn_layer_backward_terms(g.row_ptr, g.col_idx, H64, beta, dY64)
    tb = tb if tb > 0 else 1.0
    eh, eb = term_err(dH, dH_ref, tH), abs(float(dbeta.item()) - dbeta_ref) / tb
    say(f"  edge-array route: dH err {eh:.3e} dbeta err {eb:.3e}")
    assert eh < 1e-5 and eb < 1e-5
    fused_ok = B.lib().ftc_agnn_layer_backward_fused_workspace_bytes(n, g.nnz, D) > 0 and (D * Hd.element_size()) % 16 == 0
    if fused_ok:
        row_z = torch.empty(n, dtype=F32, device="cuda")
        Y = B.ftc_agnn_layer(dg, win, Hd, beta=beta, row_z=row_z)
        dH2, dbeta2 = B.ftc_agnn_layer_backward_fused(dg, win, Hd, row_z, Y, dYd, beta=beta)
        eh2, eb2 = term_err(dH2, dH_ref, tH), abs(float(dbeta2.item()) - dbeta_ref) / tb
        say(f"  single-pass route: dH err {eh2:.3e} dbeta err {eb2:.3e}")
        assert eh2 < 1e-5 and eb2 < 1e-5
