"""ctypes binding of libftc.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/ftc.h).  Tensors
are torch CUDA tensors used purely as device buffers; outputs and workspaces are
allocated with torch.empty and handed to the library as raw pointers.  All work is
enqueued on torch's current stream.  There is no CPU or PyTorch fallback: if the shared
library is missing, lib() raises.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libftc.so")

FTC_F32, FTC_F16, FTC_BF16 = 0, 1, 2
FTC_PATH_AUTO, FTC_PATH_VALU, FTC_PATH_MFMA = 0, 1, 2
FTC_OK, FTC_EINVAL, FTC_EUNSUPPORTED, FTC_EALIGN, FTC_EWORKSPACE, FTC_EHIP = 0, -1, -2, -3, -4, -5

_DTYPES = {torch.float32: FTC_F32, torch.float16: FTC_F16, torch.bfloat16: FTC_BF16}

_I, _P, _Z, _F = C.c_int32, C.c_void_p, C.c_size_t, C.c_float

# (restype, argtypes) of every export, in the order of include/ftc.h; with these set, ctypes
# rejects a call with the wrong number of arguments instead of passing garbage.
_SIGNATURES = {
    "ftc_version": (_I, []),
    "ftc_last_error": (C.c_char_p, []),
    "ftc_validate_csr": (_I, [_P, _P, _P]),
    "ftc_build_windows_workspace_bytes": (_Z, [_I, _I, _I, _I]),
    "ftc_build_windows": (_I, [_P, _P, _P, _Z, _P]),
    "ftc_build_windows_concurrent": (_I, [_P, _P, _P, _Z, _P, _P]),
    "ftc_gcn_norm": (_I, [_P, _P, _P, _P, _P]),
    "ftc_spmm_workspace_bytes": (_Z, [_I, _I, _I]),
    "ftc_spmm": (_I, [_P, _P, _P, _P, _I, _I, _I, _P, _I, _I, _P, _I, _I, _P, _Z, _P]),
    "ftc_spmm_noalloc": (_I, [_P, _P, _P, _P, _I, _I, _I, _P, _I, _I, _P, _I, _I, _P]),
    "ftc_sddmm_workspace_bytes": (_Z, [_I, _I, _I]),
    "ftc_sddmm": (_I, [_P, _P, _P, _P, _I, _I, _I, _P, _P, _F, _I, _P, _I, _P, _Z, _P]),
    "ftc_row_rnorm": (_I, [_I, _P, _I, _I, _I, _P, _P]),
    "ftc_edge_softmax_workspace_bytes": (_Z, [_I, _I]),
    "ftc_edge_softmax": (_I, [_P, _P, _P, _P, _P, _Z, _P]),
    "ftc_update_gemm": (_I, [_I, _P, _I, _I, _I, _P, _I, _P, _I, _I, _P, _I, _P]),
    "ftc_gcn_layer_workspace_bytes": (_Z, [_I, _I, _I, _I]),
    "ftc_gcn_layer": (_I, [_P, _P, _P, _P, _P, _I, _I, _I, _P, _I, _I, _P, _I, _I, _I, _P, _Z, _P]),
    "ftc_agnn_layer_workspace_bytes": (_Z, [_I, _I, _I]),
    "ftc_agnn_layer": (_I, [_P, _P, _P, _I, _I, _I, _F, _P, _I, _I, _P, _P, _P, _I, _I, _P, _Z, _P]),
    "ftc_transpose_index": (_I, [_P, _P, _P, _P, _P]),
    "ftc_edge_softmax_backward": (_I, [_P, _P, _P, _P, _P, _P, _Z, _P]),
    "ftc_weight_grad_workspace_bytes": (_Z, [_I, _I, _I]),
    "ftc_weight_grad": (_I, [_I, _P, _I, _I, _I, _P, _I, _I, _P, _P, _Z, _P]),
    "ftc_update_gemm_backward_workspace_bytes": (_Z, [_I, _I, _I]),
    "ftc_update_gemm_backward": (_I, [_I, _P, _I, _I, _I, _P, _I, _P, _I, _I, _P, _I, _P, _I, _I, _P, _P, _Z, _P]),
    "ftc_gcn_layer_backward_workspace_bytes": (_Z, [_I, _I, _I, _I]),
    "ftc_gcn_layer_backward": (_I, [_P, _P, _P, _P, _P, _I, _I, _I, _P, _I, _P, _I, _I, _P, _I, _P, _I, _P, _I, _P,
                                    _Z, _P]),
    "ftc_agnn_layer_backward_workspace_bytes": (_Z, [_I, _I, _I]),
    "ftc_agnn_layer_backward": (_I, [_P, _P, _P, _P, _I, _I, _I, _F, _P, _P, _I, _P, _I, _I, _P, _I, _P, _Z, _P]),
    "ftc_agnn_layer_backward_fused_workspace_bytes": (_Z, [_I, _I, _I]),
    "ftc_agnn_layer_backward_fused": (_I, [_P, _P, _P, _I, _I, _I, _F, _P, _P, _I, _I, _P, _I, _P, _I, _I, _P, _P, _P, _Z, _P]),
    "ftc_reorder_workspace_bytes": (_Z, [_I, _I]),
    "ftc_degree_order": (_I, [_P, _I, _P, _P, _P, _Z, _P]),
    "ftc_order_by_key": (_I, [_I, _P, _P, _P, _P, _P, _Z, _P]),
    "ftc_label_propagation": (_I, [_P, _I, _P, _P, _Z, _P]),
    "ftc_permute_graph": (_I, [_P, _P, _P, _P, _P, _P, _P, _Z, _P]),
    "ftc_permute_rows": (_I, [_I, _P, _I, _I, _I, _P, _P, _I, _P]),
    "ftc_degree_stats": (_I, [_P, _P, _P]),
    "ftc_plan_graph": (_I, [_I, _I, C.c_int64, C.c_int64, _I, _I, _P]),
}
EXPORTS = list(_SIGNATURES)


class FtcError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libftc error {code}: {msg}")
        self.code = code


class ftc_csr(C.Structure):
    _fields_ = [("n", C.c_int32), ("nnz", C.c_int32), ("row_ptr", C.c_void_p), ("col_idx", C.c_void_p)]


class ftc_windows(C.Structure):
    _fields_ = [("blk_h", C.c_int32), ("blk_w", C.c_int32), ("n_windows", C.c_int32),
                ("edge_to_row", C.c_void_p), ("edge_to_col", C.c_void_p),
                ("block_partition", C.c_void_p), ("win_col_ptr", C.c_void_p),
                ("win_cols", C.c_void_p), ("summary", C.c_void_p)]


_lib = None


def lib():
    """Load libftc.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _check(code):
    if code != FTC_OK:
        raise FtcError(code, lib().ftc_last_error().decode())


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dt(t):
    return _DTYPES[t.dtype]


class Graph:
    """Device CSR adjacency (int32) plus its C descriptor."""

    def __init__(self, row_ptr, col_idx):
        assert row_ptr.dtype == torch.int32 and col_idx.dtype == torch.int32
        assert row_ptr.is_cuda and col_idx.is_cuda and row_ptr.is_contiguous() and col_idx.is_contiguous()
        self.row_ptr, self.col_idx = row_ptr, col_idx
        self.n = row_ptr.numel() - 1
        self.nnz = col_idx.numel()
        self.c = ftc_csr(self.n, self.nnz, row_ptr.data_ptr(), col_idx.data_ptr() if self.nnz else 0)

    @staticmethod
    def from_numpy(row_ptr, col_idx, device="cuda"):
        return Graph(torch.from_numpy(row_ptr).to(device=device, dtype=torch.int32),
                     torch.from_numpy(col_idx).to(device=device, dtype=torch.int32))


class Windows:
    """Device arrays of the sparse graph transformation plus their C descriptor."""

    def __init__(self, g, blk_h=16, blk_w=8):
        dev = g.row_ptr.device
        self.blk_h, self.blk_w = blk_h, blk_w
        self.n_windows = (g.n + blk_h - 1) // blk_h
        i32 = dict(dtype=torch.int32, device=dev)
        self.edge_to_row = torch.empty(g.nnz, **i32)
        self.edge_to_col = torch.empty(g.nnz, **i32)
        self.block_partition = torch.empty(self.n_windows, **i32)
        self.win_col_ptr = torch.empty(self.n_windows + 1, **i32)
        self.win_cols = torch.empty(g.nnz, **i32)
        self.summary = torch.empty(2, dtype=torch.int64, device=dev)
        self.c = ftc_windows(blk_h, blk_w, self.n_windows, self.edge_to_row.data_ptr(),
                             self.edge_to_col.data_ptr(), self.block_partition.data_ptr(),
                             self.win_col_ptr.data_ptr(), self.win_cols.data_ptr(),
                             self.summary.data_ptr())


def _workspace(nbytes, device):
    # torch's caching allocator returns 512-byte aligned blocks
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _wref(w):
    return C.byref(w.c) if w is not None else None


def ftc_version():
    return lib().ftc_version()


def ftc_validate_csr(g):
    flag = torch.empty(1, dtype=torch.int32, device=g.row_ptr.device)
    _check(lib().ftc_validate_csr(C.byref(g.c), _ptr(flag), _stream()))
    return flag


class ftc_side_streams(C.Structure):
    _fields_ = [("stream", C.c_void_p * 3), ("fork", C.c_void_p), ("join", C.c_void_p * 3)]


class SideStreams:
    """Three streams and four events for ftc_build_windows_concurrent, created through torch (device plumbing
    only) on the current device at the default priority; keeps them alive as long as the object lives."""

    def __init__(self):
        self.streams = [torch.cuda.Stream() for _ in range(3)]
        self.events = [torch.cuda.Event(enable_timing=False) for _ in range(4)]
        for ev, st in zip(self.events, [torch.cuda.current_stream()] + self.streams):
            ev.record(st)              # torch creates the event handle at its first record
        self.c = ftc_side_streams()
        for i in range(3):
            self.c.stream[i] = self.streams[i].cuda_stream
            self.c.join[i] = self.events[1 + i].cuda_event
        self.c.fork = self.events[0].cuda_event


def ftc_build_windows(g, blk_h=16, blk_w=8, out=None, ws=None):
    w = out if out is not None else Windows(g, blk_h, blk_w)
    if ws is None:
        ws = _workspace(lib().ftc_build_windows_workspace_bytes(g.n, g.nnz, w.c.blk_h, w.c.blk_w), g.row_ptr.device)
    _check(lib().ftc_build_windows(C.byref(g.c), C.byref(w.c), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
    return w


def ftc_build_windows_concurrent(g, side, blk_h=16, blk_w=8, out=None, ws=None):
    """side: a SideStreams (or None: the same as ftc_build_windows)."""
    w = out if out is not None else Windows(g, blk_h, blk_w)
    if ws is None:
        ws = _workspace(lib().ftc_build_windows_workspace_bytes(g.n, g.nnz, w.c.blk_h, w.c.blk_w), g.row_ptr.device)
    _check(lib().ftc_build_windows_concurrent(C.byref(g.c), C.byref(w.c), _ptr(ws), C.c_size_t(ws.numel()),
                                              C.byref(side.c) if side is not None else None, _stream()))
    return w


def ftc_gcn_norm(g, w=None, want_vals=True, want_dinv=True):
    dev = g.row_ptr.device
    vals = torch.empty(g.nnz, dtype=torch.float32, device=dev) if want_vals else None
    dinv = torch.empty(g.n, dtype=torch.float32, device=dev) if want_dinv else None
    _check(lib().ftc_gcn_norm(C.byref(g.c), _wref(w), _ptr(vals), _ptr(dinv), _stream()))
    return vals, dinv


def ftc_spmm(g, w, vals, X, out=None, out_dtype=torch.float32, relu=False, path=FTC_PATH_AUTO, ws=None,
             out_scale=None):
    D = X.shape[1]
    if out is None:
        out = torch.empty((g.n, D), dtype=out_dtype, device=X.device)
    if ws is None:
        ws = _workspace(lib().ftc_spmm_workspace_bytes(g.n, g.nnz, D), X.device)
    _check(lib().ftc_spmm(C.byref(g.c), _wref(w), _ptr(vals), _ptr(X), C.c_int32(X.stride(0)),
                          C.c_int32(_dt(X)), C.c_int32(D), _ptr(out), C.c_int32(out.stride(0)),
                          C.c_int32(_dt(out)), _ptr(out_scale), C.c_int32(1 if relu else 0), C.c_int32(path),
                          _ptr(ws), C.c_size_t(ws.numel()), _stream()))
    return out


def ftc_spmm_noalloc(g, w, vals, X, out, relu=False, path=FTC_PATH_AUTO, out_scale=None):
    """ftc_spmm on the library's built-in scratch buffer; `out` is the caller's (nothing is allocated here)."""
    D = X.shape[1]
    _check(lib().ftc_spmm_noalloc(C.byref(g.c), _wref(w), _ptr(vals), _ptr(X), C.c_int32(X.stride(0)),
                                  C.c_int32(_dt(X)), C.c_int32(D), _ptr(out), C.c_int32(out.stride(0)),
                                  C.c_int32(_dt(out)), _ptr(out_scale), C.c_int32(1 if relu else 0), C.c_int32(path),
                                  _stream()))
    return out


def ftc_sddmm(g, w, X, Y, row_scale=None, col_scale=None, alpha=1.0, out=None, path=FTC_PATH_AUTO, ws=None,
              cosine=False):
    D = X.shape[1]
    assert Y.shape[1] == D and X.stride(0) == Y.stride(0) and X.dtype == Y.dtype
    if out is None:
        out = torch.empty(g.nnz, dtype=torch.float32, device=X.device)
    if ws is None:
        ws = _workspace(lib().ftc_sddmm_workspace_bytes(g.n, g.nnz, D), X.device)
    _check(lib().ftc_sddmm(C.byref(g.c), _wref(w), _ptr(X), _ptr(Y), C.c_int32(X.stride(0)),
                           C.c_int32(_dt(X)), C.c_int32(D), _ptr(row_scale), _ptr(col_scale),
                           C.c_float(alpha), C.c_int32(1 if cosine else 0), _ptr(out), C.c_int32(path), _ptr(ws),
                           C.c_size_t(ws.numel()), _stream()))
    return out


def ftc_row_rnorm(H, out=None):
    if out is None:
        out = torch.empty(H.shape[0], dtype=torch.float32, device=H.device)
    _check(lib().ftc_row_rnorm(C.c_int32(H.shape[0]), _ptr(H), C.c_int32(H.stride(0)), C.c_int32(_dt(H)),
                               C.c_int32(H.shape[1]), _ptr(out), _stream()))
    return out


def ftc_edge_softmax(g, w, e_in, out=None, ws=None):
    if out is None:
        out = torch.empty_like(e_in)
    if ws is None:
        ws = _workspace(lib().ftc_edge_softmax_workspace_bytes(g.n, g.nnz) if w is not None else 0, e_in.device)
    _check(lib().ftc_edge_softmax(C.byref(g.c), _wref(w), _ptr(e_in), _ptr(out), _ptr(ws),
                                  C.c_size_t(ws.numel()), _stream()))
    return out


def ftc_update_gemm(X, W, out=None, out_dtype=torch.float32, relu=False, row_scale=None):
    n, d_in = X.shape
    d_out = W.shape[1]
    assert W.shape[0] == d_in and W.is_contiguous() and W.dtype == X.dtype
    if out is None:
        out = torch.empty((n, d_out), dtype=out_dtype, device=X.device)
    _check(lib().ftc_update_gemm(C.c_int32(n), _ptr(X), C.c_int32(X.stride(0)), C.c_int32(_dt(X)),
                                 C.c_int32(d_in), _ptr(W), C.c_int32(d_out), _ptr(out),
                                 C.c_int32(out.stride(0)), C.c_int32(_dt(out)), _ptr(row_scale),
                                 C.c_int32(1 if relu else 0), _stream()))
    return out


def ftc_gcn_layer(g, w, vals, X, W, relu=False, out=None, out_dtype=torch.float32, path=FTC_PATH_AUTO,
                  ws=None, dinv=None):
    n, d_in = X.shape
    d_out = W.shape[1]
    assert W.shape[0] == d_in and W.is_contiguous() and W.dtype == X.dtype
    if out is None:
        out = torch.empty((n, d_out), dtype=out_dtype, device=X.device)
    if ws is None:
        ws = _workspace(lib().ftc_gcn_layer_workspace_bytes(g.n, g.nnz, d_in, d_out), X.device)
    _check(lib().ftc_gcn_layer(C.byref(g.c), _wref(w), _ptr(vals), _ptr(dinv), _ptr(X), C.c_int32(X.stride(0)),
                               C.c_int32(_dt(X)), C.c_int32(d_in), _ptr(W), C.c_int32(d_out),
                               C.c_int32(1 if relu else 0), _ptr(out), C.c_int32(out.stride(0)),
                               C.c_int32(_dt(out)), C.c_int32(path), _ptr(ws), C.c_size_t(ws.numel()),
                               _stream()))
    return out


def ftc_agnn_layer(g, w, H, beta=1.0, out=None, out_dtype=torch.float32, edge_p=None, path=FTC_PATH_AUTO,
                   ws=None, row_z=None, out_f32=None):
    n, D = H.shape
    if out is None:
        out = torch.empty((n, D), dtype=out_dtype, device=H.device)
    if ws is None:
        ws = _workspace(lib().ftc_agnn_layer_workspace_bytes(g.n, g.nnz, D), H.device)
    _check(lib().ftc_agnn_layer(C.byref(g.c), _wref(w), _ptr(H), C.c_int32(H.stride(0)), C.c_int32(_dt(H)),
                                C.c_int32(D), C.c_float(beta), _ptr(out), C.c_int32(out.stride(0)),
                                C.c_int32(_dt(out)), _ptr(edge_p), _ptr(row_z), _ptr(out_f32),
                                C.c_int32(out_f32.stride(0) if out_f32 is not None else 0), C.c_int32(path), _ptr(ws),
                                C.c_size_t(ws.numel()), _stream()))
    return out


# ---- backward pass (gradients are fp32 tensors) ----------------------------------------------------
def ftc_transpose_index(g, w=None):
    T = torch.empty(g.nnz, dtype=torch.int32, device=g.row_ptr.device)
    flag = torch.empty(1, dtype=torch.int32, device=g.row_ptr.device)
    _check(lib().ftc_transpose_index(C.byref(g.c), _wref(w), _ptr(T), _ptr(flag), _stream()))
    return T, flag


def ftc_edge_softmax_backward(g, w, p, dp, out=None, ws=None):
    if out is None:
        out = torch.empty_like(dp)
    if ws is None:
        ws = _workspace(lib().ftc_edge_softmax_workspace_bytes(g.n, g.nnz), dp.device)
    _check(lib().ftc_edge_softmax_backward(C.byref(g.c), _wref(w), _ptr(p), _ptr(dp), _ptr(out), _ptr(ws),
                                           C.c_size_t(ws.numel()), _stream()))
    return out


def ftc_weight_grad(X, G, ws=None):
    n, d_in = X.shape
    d_out = G.shape[1]
    assert G.dtype == torch.float32 and G.shape[0] == n
    dW = torch.empty((d_in, d_out), dtype=torch.float32, device=X.device)
    if ws is None:
        ws = _workspace(lib().ftc_weight_grad_workspace_bytes(n, d_in, d_out), X.device)
    _check(lib().ftc_weight_grad(C.c_int32(n), _ptr(X), C.c_int32(X.stride(0)), C.c_int32(_dt(X)), C.c_int32(d_in),
                                 _ptr(G), C.c_int32(G.stride(0)), C.c_int32(d_out), _ptr(dW), _ptr(ws),
                                 C.c_size_t(ws.numel()), _stream()))
    return dW


def ftc_update_gemm_backward(X, W, dZ, Z=None, want_dX=True, dx_dtype=torch.float32, dX=None, ws=None):
    n, d_in = X.shape
    d_out = W.shape[1]
    assert dZ.dtype == torch.float32 and dZ.shape == (n, d_out)
    if dX is None and want_dX:
        dX = torch.empty((n, d_in), dtype=dx_dtype, device=X.device)
    dW = torch.empty((d_in, d_out), dtype=torch.float32, device=X.device)
    if ws is None:
        ws = _workspace(lib().ftc_update_gemm_backward_workspace_bytes(n, d_in, d_out), X.device)
    _check(lib().ftc_update_gemm_backward(
        C.c_int32(n), _ptr(X), C.c_int32(X.stride(0)), C.c_int32(_dt(X)), C.c_int32(d_in), _ptr(W), C.c_int32(d_out),
        _ptr(Z), C.c_int32(Z.stride(0) if Z is not None else 0), C.c_int32(_dt(Z) if Z is not None else 0), _ptr(dZ),
        C.c_int32(dZ.stride(0)), _ptr(dX), C.c_int32(dX.stride(0) if dX is not None else 0),
        C.c_int32(_dt(dX) if dX is not None else 0), _ptr(dW), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
    return dX, dW


def ftc_gcn_layer_backward(gT, wT, valsT, X, W, dY, Y=None, dinv=None, want_dX=True, path=FTC_PATH_AUTO, ws=None):
    n, d_in = X.shape
    d_out = W.shape[1]
    assert dY.dtype == torch.float32 and dY.shape == (n, d_out)
    dX = torch.empty((n, d_in), dtype=torch.float32, device=X.device) if want_dX else None
    dW = torch.empty((d_in, d_out), dtype=torch.float32, device=X.device)
    if ws is None:
        ws = _workspace(lib().ftc_gcn_layer_backward_workspace_bytes(gT.n, gT.nnz, d_in, d_out), X.device)
    _check(lib().ftc_gcn_layer_backward(
        C.byref(gT.c), _wref(wT), _ptr(valsT), _ptr(dinv), _ptr(X), C.c_int32(X.stride(0)), C.c_int32(_dt(X)),
        C.c_int32(d_in), _ptr(W), C.c_int32(d_out), _ptr(Y), C.c_int32(Y.stride(0) if Y is not None else 0),
        C.c_int32(_dt(Y) if Y is not None else 0), _ptr(dY), C.c_int32(dY.stride(0)), _ptr(dX),
        C.c_int32(dX.stride(0) if dX is not None else 0), _ptr(dW), C.c_int32(path), _ptr(ws), C.c_size_t(ws.numel()),
        _stream()))
    return dX, dW


def ftc_agnn_layer_backward(g, w, T, H, p, dY, beta=1.0, dH=None, dh_dtype=torch.float32, dbeta=None,
                            path=FTC_PATH_AUTO, ws=None):
    n, D = H.shape
    assert dY.dtype == H.dtype and dY.shape == H.shape and dY.stride(0) == H.stride(0)
    if dH is None:
        dH = torch.empty((n, D), dtype=dh_dtype, device=H.device)
    if dbeta is None:
        dbeta = torch.empty(1, dtype=torch.float32, device=H.device)
    if ws is None:
        ws = _workspace(lib().ftc_agnn_layer_backward_workspace_bytes(g.n, g.nnz, D), H.device)
    _check(lib().ftc_agnn_layer_backward(
        C.byref(g.c), _wref(w), _ptr(T), _ptr(H), C.c_int32(H.stride(0)), C.c_int32(_dt(H)), C.c_int32(D),
        C.c_float(beta), _ptr(p), _ptr(dY), C.c_int32(dY.stride(0)), _ptr(dH), C.c_int32(dH.stride(0)),
        C.c_int32(_dt(dH)), _ptr(dbeta), C.c_int32(path), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
    return dH, dbeta


def ftc_agnn_layer_backward_fused(g, w, H, row_z, Y, dY, beta=1.0, dH=None, dh_dtype=torch.float32, dbeta=None, ws=None,
                                  pattern_flag=None):
    n, D = H.shape
    assert dY.dtype == H.dtype and dY.shape == H.shape and dY.stride(0) == H.stride(0) and Y.shape == H.shape
    if dH is None:
        dH = torch.empty((n, D), dtype=dh_dtype, device=H.device)
    if dbeta is None:
        dbeta = torch.empty(1, dtype=torch.float32, device=H.device)
    if ws is None:
        ws = _workspace(lib().ftc_agnn_layer_backward_fused_workspace_bytes(g.n, g.nnz, D), H.device)
    _check(lib().ftc_agnn_layer_backward_fused(
        C.byref(g.c), _wref(w), _ptr(H), C.c_int32(H.stride(0)), C.c_int32(_dt(H)), C.c_int32(D), C.c_float(beta),
        _ptr(row_z), _ptr(Y), C.c_int32(Y.stride(0)), C.c_int32(_dt(Y)), _ptr(dY), C.c_int32(dY.stride(0)), _ptr(dH),
        C.c_int32(dH.stride(0)), C.c_int32(_dt(dH)), _ptr(dbeta), _ptr(pattern_flag), _ptr(ws), C.c_size_t(ws.numel()),
        _stream()))
    return dH, dbeta


# ---- locality reordering ------------------------------------------------------------------------------
FTC_ORDER_DEGREE, FTC_ORDER_DEGREE_CLASSES, FTC_ORDER_COMMUNITIES = 0, 1, 2


def ftc_degree_order(g, mode=FTC_ORDER_DEGREE, ws=None):
    dev = g.row_ptr.device
    perm = torch.empty(g.n, dtype=torch.int32, device=dev)
    inv = torch.empty(g.n, dtype=torch.int32, device=dev)
    if ws is None:
        ws = _workspace(lib().ftc_reorder_workspace_bytes(g.n, g.nnz), dev)
    _check(lib().ftc_degree_order(C.byref(g.c), C.c_int32(mode), _ptr(perm), _ptr(inv), _ptr(ws),
                                  C.c_size_t(ws.numel()), _stream()))
    return perm, inv


def ftc_order_by_key(keys, ws=None):
    """Returns (perm, inv, flag): ascending keys, ties by id."""
    n = keys.numel()
    dev = keys.device
    perm = torch.empty(n, dtype=torch.int32, device=dev)
    inv = torch.empty(n, dtype=torch.int32, device=dev)
    flag = torch.empty(1, dtype=torch.int32, device=dev)
    if ws is None:
        ws = _workspace(lib().ftc_reorder_workspace_bytes(n, 0), dev)
    _check(lib().ftc_order_by_key(C.c_int32(n), _ptr(keys), _ptr(perm), _ptr(inv), _ptr(flag), _ptr(ws),
                                  C.c_size_t(ws.numel()), _stream()))
    return perm, inv, flag


def ftc_label_propagation(g, rounds=10, ws=None):
    dev = g.row_ptr.device
    labels = torch.empty(g.n, dtype=torch.int32, device=dev)
    if ws is None:
        ws = _workspace(lib().ftc_reorder_workspace_bytes(g.n, g.nnz), dev)
    _check(lib().ftc_label_propagation(C.byref(g.c), C.c_int32(rounds), _ptr(labels), _ptr(ws), C.c_size_t(ws.numel()),
                                       _stream()))
    return labels


def ftc_permute_graph(g, perm, inv, ws=None):
    """Returns (relabelled Graph, flag tensor: 0 if (perm, inv) is a permutation and its inverse)."""
    dev = g.row_ptr.device
    row_ptr = torch.empty(g.n + 1, dtype=torch.int32, device=dev)
    col_idx = torch.empty(g.nnz, dtype=torch.int32, device=dev)
    flag = torch.empty(1, dtype=torch.int32, device=dev)
    if ws is None:
        ws = _workspace(lib().ftc_reorder_workspace_bytes(g.n, g.nnz), dev)
    _check(lib().ftc_permute_graph(C.byref(g.c), _ptr(perm), _ptr(inv), _ptr(row_ptr), _ptr(col_idx), _ptr(flag),
                                   _ptr(ws), C.c_size_t(ws.numel()), _stream()))
    return Graph(row_ptr, col_idx), flag


def ftc_permute_rows(X, index, out=None):
    n, D = X.shape
    if out is None:
        out = torch.empty((n, D), dtype=X.dtype, device=X.device)
    _check(lib().ftc_permute_rows(C.c_int32(n), _ptr(X), C.c_int32(X.stride(0)), C.c_int32(_dt(X)), C.c_int32(D),
                                  _ptr(index), _ptr(out), C.c_int32(out.stride(0)), _stream()))
    return out


# ---- per-graph plan -------------------------------------------------------------------------------------
FTC_ORDER_NONE = -1


class ftc_plan(C.Structure):
    _fields_ = [("skew", C.c_double), ("reuse", C.c_double), ("reorder", C.c_int32), ("agnn_single_pass", C.c_int32),
                ("agnn_backward_single_pass", C.c_int32), ("spmm_mfma_windows", C.c_int32),
                ("sddmm_mfma_windows", C.c_int32), ("mfma_min_reuse", C.c_float)]


def ftc_degree_stats(g):
    stats = torch.empty(2, dtype=torch.int64, device=g.row_ptr.device)
    _check(lib().ftc_degree_stats(C.byref(g.c), _ptr(stats), _stream()))
    return stats


def ftc_plan_graph(n, nnz, sum_deg_sq, sum_uniq, D, dtype):
    """Host-only: the per-graph choices as a dict (dtype: a torch dtype)."""
    plan = ftc_plan()
    _check(lib().ftc_plan_graph(C.c_int32(n), C.c_int32(nnz), C.c_int64(int(sum_deg_sq)), C.c_int64(int(sum_uniq)),
                                C.c_int32(D), C.c_int32(_DTYPES[dtype]), C.byref(plan)))
    return {name: getattr(plan, name) for name, _ in ftc_plan._fields_}
