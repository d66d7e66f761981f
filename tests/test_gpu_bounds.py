"""No kernel writes outside its output arrays: every output lives in the middle of a larger buffer
whose guard zones (and, for strided matrices, padding columns) must keep their sentinel."""
import numpy as np
import pytest
import torch

import synth
from parity import dev_graph
from paper_2412_12218_amd import binding as B

pytestmark = pytest.mark.gpu
F32, F16, BF16 = torch.float32, torch.float16, torch.bfloat16
GUARD = 4096


class Guarded:
    """A tensor view of `shape` (optionally with `pad` extra columns) inside a sentinel-filled buffer."""

    def __init__(self, shape, dtype, pad=0, sentinel=None):
        rows = shape[0]
        cols = (shape[1] + pad) if len(shape) == 2 else 1
        n = rows * cols
        if sentinel is None:
            sentinel = -12345.0 if dtype.is_floating_point else -77
        self.sentinel = sentinel
        self.buf = torch.full((n + 2 * GUARD,), self.sentinel, dtype=dtype, device="cuda")
        body = self.buf[GUARD:GUARD + n]
        self.full = body.view(rows, cols) if len(shape) == 2 else body
        self.view = self.full[:, :shape[1]] if len(shape) == 2 else body
        self.pad = pad

    def check(self):
        s = torch.tensor(self.sentinel, dtype=self.buf.dtype, device="cuda")
        assert torch.all(self.buf[:GUARD] == s) and torch.all(self.buf[-GUARD:] == s), "guard zone overwritten"
        if self.pad:
            assert torch.all(self.full[:, -self.pad:] == s), "padding columns overwritten"
        assert not torch.any(self.view == s), "part of the output was never written"


def graphs():
    rng = np.random.default_rng(9)
    n = 1000 + 7
    rows = [rng.integers(0, n, size=rng.integers(1, 30)) for _ in range(n)]
    rows[3] = rng.integers(0, n, size=6000)      # a window for the bitmap kernel, rows cut by wave ranges
    rows[500] = rng.integers(0, n, size=1500)
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum([len(r) for r in rows])
    hub = synth.Graph(n, row_ptr, np.concatenate(rows).astype(np.int32))
    return [hub, synth.config_graph(5, 1 / 64)]


@pytest.mark.parametrize("gi", [0, 1])
def test_build_windows_stays_in_bounds(gi):
    g = graphs()[gi]
    dg = dev_graph(g)
    w = B.Windows(dg)
    n_win = w.n_windows
    guards = {name: Guarded((size,), torch.int32) for name, size in
              (("edge_to_row", g.nnz), ("edge_to_col", g.nnz), ("block_partition", n_win),
               ("win_col_ptr", n_win + 1), ("win_cols", g.nnz))}
    summ = Guarded((2,), torch.int64)
    w.c = B.ftc_windows(16, 8, n_win, *(guards[k].view.data_ptr() for k in
                                         ("edge_to_row", "edge_to_col", "block_partition", "win_col_ptr", "win_cols")),
                        summ.view.data_ptr())
    nbytes = B.lib().ftc_build_windows_workspace_bytes(g.n, g.nnz, 16, 8)
    ws = Guarded((nbytes,), torch.uint8, sentinel=0)   # workspace: only the guard zones are checked
    B._check(B.lib().ftc_build_windows(B.C.byref(dg.c), B.C.byref(w.c), B._ptr(ws.view), B.C.c_size_t(nbytes),
                                       B._stream()))
    torch.cuda.synchronize()
    for name in ("edge_to_row", "edge_to_col", "block_partition", "win_col_ptr"):
        guards[name].check()
    uniq = int(summ.view[0].item())
    wc = guards["win_cols"]
    assert torch.all(wc.buf[:GUARD] == -77) and torch.all(wc.buf[-GUARD:] == -77)
    assert torch.all(wc.view[uniq:] == -77) and not torch.any(wc.view[:uniq] == -77)
    assert torch.all(ws.buf[:GUARD] == 0) and torch.all(ws.buf[-GUARD:] == 0)


@pytest.mark.parametrize("gi", [0, 1])
@pytest.mark.parametrize("dtype,D,pad", [(F16, 32, 0), (F16, 32, 8), (BF16, 64, 0), (F32, 16, 4), (F16, 8, 8),
                                         (F16, 20, 3)])
@pytest.mark.parametrize("path", [B.FTC_PATH_AUTO, B.FTC_PATH_MFMA])
def test_spmm_sddmm_softmax_stay_in_bounds(gi, dtype, D, pad, path):
    if path == B.FTC_PATH_MFMA and (dtype == F32 or D % 8 != 0 or (pad % 8) != 0):
        pytest.skip("matrix-core path needs 16-bit features with aligned rows")
    g = graphs()[gi]
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    X = torch.randn((g.n, D + pad), device="cuda").to(dtype)[:, :D]
    vals = torch.rand(g.nnz, device="cuda")
    for out_dtype in (F32, F16):
        out = Guarded((g.n, D), out_dtype, pad=pad if out_dtype == F32 else (pad + 7) // 8 * 8)
        ws = Guarded((max(B.lib().ftc_spmm_workspace_bytes(g.n, g.nnz, D), 256),), torch.uint8, sentinel=0)
        B.ftc_spmm(dg, win, vals, X, out=out.view, path=path, ws=ws.view)
        torch.cuda.synchronize()
        out.check()
        assert torch.all(ws.buf[:GUARD] == 0) and torch.all(ws.buf[-GUARD:] == 0)
    s = Guarded((g.nnz,), F32)
    B.ftc_sddmm(dg, win, X, X, None, None, 1.0, out=s.view, path=path)
    torch.cuda.synchronize()
    s.check()
    p = Guarded((g.nnz,), F32)
    B.ftc_edge_softmax(dg, win, s.view, out=p.view)
    torch.cuda.synchronize()
    p.check()


@pytest.mark.parametrize("dtype,D", [(F16, 32), (BF16, 64), (F32, 16), (F16, 8)])
def test_layers_stay_in_bounds(dtype, D):
    g = graphs()[0]
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    H = torch.randn((g.n, D), device="cuda").to(dtype)
    out = Guarded((g.n, D), F32)
    B.ftc_agnn_layer(dg, win, H, beta=1.0, out=out.view)
    torch.cuda.synchronize()
    out.check()
    p = Guarded((g.nnz,), F32)
    out2 = Guarded((g.n, D), F16)
    B.ftc_agnn_layer(dg, win, H, beta=1.0, out=out2.view, edge_p=p.view)
    torch.cuda.synchronize()
    out2.check()
    p.check()
    W = torch.randn((D, 16), device="cuda").to(dtype)
    vals = torch.rand(g.nnz, device="cuda")
    out3 = Guarded((g.n, 16), F32)
    B.ftc_gcn_layer(dg, win, vals, H, W, relu=False, out=out3.view)
    torch.cuda.synchronize()
    out3.check()
    z = Guarded((g.n, 16), F16, pad=8)
    B.ftc_update_gemm(H, W, out=z.view)
    torch.cuda.synchronize()
    z.check()
    r = Guarded((g.n,), F32)
    B.ftc_row_rnorm(H, out=r.view)
    torch.cuda.synchronize()
    r.check()


def symmetric_graph():
    """The hub graph of graphs(), symmetrised (ascending, duplicate-free rows) for the backward pass."""
    import scipy.sparse as sp
    g = graphs()[0]
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    A = sp.csr_matrix((np.ones(g.nnz), (rows, g.col_idx)), shape=(g.n, g.n))
    A = (A + A.T).tocsr()
    A.sum_duplicates()
    A.sort_indices()
    return synth.Graph(g.n, A.indptr.astype(np.int32), A.indices.astype(np.int32))


def guarded_ws(nbytes):
    return Guarded((max(int(nbytes), 256),), torch.uint8, sentinel=0)


def ws_intact(ws):
    assert torch.all(ws.buf[:GUARD] == 0) and torch.all(ws.buf[-GUARD:] == 0), "workspace guard zone overwritten"


@pytest.mark.parametrize("dtype,D", [(F16, 32), (BF16, 24), (F32, 16), (F16, 64)])
def test_agnn_training_pair_stays_in_bounds(dtype, D):
    """Single-pass forward with its two extra outputs, both backward routes, the transposed index and
    the softmax backward: outputs and workspaces between guard zones."""
    g = symmetric_graph()
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    L = B.lib()
    H = torch.randn((g.n, D), device="cuda").to(dtype)
    dY = torch.randn((g.n, D), device="cuda").to(dtype)
    out, z = Guarded((g.n, D), dtype), Guarded((g.n,), F32)
    y32 = Guarded((g.n, D), F32, pad=(-D) % 4)
    ws = guarded_ws(L.ftc_agnn_layer_workspace_bytes(g.n, g.nnz, D))
    B.ftc_agnn_layer(dg, win, H, beta=1.0, out=out.view, row_z=z.view, out_f32=y32.full, ws=ws.view)
    torch.cuda.synchronize()
    out.check(); z.check(); ws_intact(ws)
    assert torch.all(y32.buf[:GUARD] == y32.sentinel) and torch.all(y32.buf[-GUARD:] == y32.sentinel)
    dH, dbeta = Guarded((g.n, D), dtype), Guarded((1,), F32)
    ws = guarded_ws(L.ftc_agnn_layer_backward_fused_workspace_bytes(g.n, g.nnz, D))
    B.ftc_agnn_layer_backward_fused(dg, win, H, z.view, y32.full[:, :D], dY, dH=dH.view, dbeta=dbeta.view, ws=ws.view)
    torch.cuda.synchronize()
    dH.check(); dbeta.check(); ws_intact(ws)
    T, flag = Guarded((g.nnz,), torch.int32), Guarded((1,), torch.int32)
    B._check(L.ftc_transpose_index(B.C.byref(dg.c), B.C.byref(win.c), B._ptr(T.view), B._ptr(flag.view), B._stream()))
    torch.cuda.synchronize()
    T.check(); flag.check()
    assert int(flag.view.item()) == 0
    p = Guarded((g.nnz,), F32)
    ws = guarded_ws(L.ftc_agnn_layer_workspace_bytes(g.n, g.nnz, D))
    B.ftc_agnn_layer(dg, win, H, beta=1.0, out=out.view, edge_p=p.view, ws=ws.view)
    dH2, dbeta2 = Guarded((g.n, D), F32, pad=3), Guarded((1,), F32)
    ws2 = guarded_ws(L.ftc_agnn_layer_backward_workspace_bytes(g.n, g.nnz, D))
    B.ftc_agnn_layer_backward(dg, win, T.view, H, p.view, dY, dH=dH2.view, dbeta=dbeta2.view, ws=ws2.view)
    torch.cuda.synchronize()
    p.check(); dH2.check(); dbeta2.check(); ws_intact(ws); ws_intact(ws2)
    ds = Guarded((g.nnz,), F32)
    ws3 = guarded_ws(L.ftc_edge_softmax_workspace_bytes(g.n, g.nnz))
    B.ftc_edge_softmax_backward(dg, win, p.view, torch.randn(g.nnz, device="cuda"), out=ds.view, ws=ws3.view)
    torch.cuda.synchronize()
    ds.check(); ws_intact(ws3)


@pytest.mark.parametrize("dtype,d_in,d_out", [(F16, 64, 16), (F32, 16, 8), (BF16, 30, 7)])
def test_dense_and_gcn_backward_stay_in_bounds(dtype, d_in, d_out):
    g = symmetric_graph()
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    L = B.lib()
    X = torch.randn((g.n, d_in), device="cuda").to(dtype)
    W = torch.randn((d_in, d_out), device="cuda").to(dtype)
    dY = torch.randn((g.n, d_out), device="cuda")
    _, dinv = B.ftc_gcn_norm(dg, win, want_vals=False)
    Y = B.ftc_gcn_layer(dg, win, None, X, W, relu=True, dinv=dinv)
    dX, dW = Guarded((g.n, d_in), F32, pad=5), Guarded((d_in, d_out), F32)
    ws = guarded_ws(L.ftc_gcn_layer_backward_workspace_bytes(g.n, g.nnz, d_in, d_out))
    B._check(L.ftc_gcn_layer_backward(
        B.C.byref(dg.c), B.C.byref(win.c), None, B._ptr(dinv), B._ptr(X), B.C.c_int32(X.stride(0)), B.C.c_int32(B._dt(X)),
        B.C.c_int32(d_in), B._ptr(W), B.C.c_int32(d_out), B._ptr(Y), B.C.c_int32(Y.stride(0)), B.C.c_int32(B._dt(Y)),
        B._ptr(dY), B.C.c_int32(dY.stride(0)), B._ptr(dX.view), B.C.c_int32(dX.view.stride(0)), B._ptr(dW.view),
        B.C.c_int32(B.FTC_PATH_AUTO), B._ptr(ws.view), B.C.c_size_t(ws.view.numel()), B._stream()))
    torch.cuda.synchronize()
    dX.check(); dW.check(); ws_intact(ws)
    dX2 = Guarded((g.n, d_in), F16, pad=3)
    ws = guarded_ws(L.ftc_update_gemm_backward_workspace_bytes(g.n, d_in, d_out))
    _, dW2 = B.ftc_update_gemm_backward(X, W, dY, Z=Y, dX=dX2.view, ws=ws.view)
    torch.cuda.synchronize()
    dX2.check(); ws_intact(ws)


@pytest.mark.parametrize("gi", [0, 1])
def test_reordering_stays_in_bounds(gi):
    g = graphs()[gi]
    dg = dev_graph(g)
    L = B.lib()
    C = B.C
    nbytes = L.ftc_reorder_workspace_bytes(g.n, g.nnz)
    perm, inv = Guarded((g.n,), torch.int32), Guarded((g.n,), torch.int32)
    ws = guarded_ws(nbytes)
    B._check(L.ftc_degree_order(C.byref(dg.c), C.c_int32(0), B._ptr(perm.view), B._ptr(inv.view), B._ptr(ws.view),
                                C.c_size_t(ws.view.numel()), B._stream()))
    torch.cuda.synchronize()
    perm.check(); inv.check(); ws_intact(ws)
    rp, ci, flag = Guarded((g.n + 1,), torch.int32), Guarded((g.nnz,), torch.int32), Guarded((1,), torch.int32)
    B._check(L.ftc_permute_graph(C.byref(dg.c), B._ptr(perm.view), B._ptr(inv.view), B._ptr(rp.view), B._ptr(ci.view),
                                 B._ptr(flag.view), B._ptr(ws.view), C.c_size_t(ws.view.numel()), B._stream()))
    torch.cuda.synchronize()
    rp.check(); ci.check(); flag.check(); ws_intact(ws)
    labels = Guarded((g.n,), torch.int32)
    B._check(L.ftc_label_propagation(C.byref(dg.c), C.c_int32(3), B._ptr(labels.view), B._ptr(ws.view),
                                     C.c_size_t(ws.view.numel()), B._stream()))
    torch.cuda.synchronize()
    labels.check(); ws_intact(ws)
    perm2, inv2, flag2 = Guarded((g.n,), torch.int32), Guarded((g.n,), torch.int32), Guarded((1,), torch.int32)
    B._check(L.ftc_order_by_key(C.c_int32(g.n), B._ptr(labels.view), B._ptr(perm2.view), B._ptr(inv2.view),
                                B._ptr(flag2.view), B._ptr(ws.view), C.c_size_t(ws.view.numel()), B._stream()))
    torch.cuda.synchronize()
    perm2.check(); inv2.check(); flag2.check(); ws_intact(ws)
    X = torch.randn((g.n, 24), device="cuda").to(F16)
    out = Guarded((g.n, 24), F16, pad=8)
    B.ftc_permute_rows(X, perm.view, out=out.view)
    torch.cuda.synchronize()
    out.check()
    stats = Guarded((2,), torch.int64)
    B._check(L.ftc_degree_stats(C.byref(dg.c), B._ptr(stats.view), B._stream()))
    torch.cuda.synchronize()
    stats.check()
