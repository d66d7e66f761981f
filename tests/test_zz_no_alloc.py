"""The entry point that allocates nothing (ftc_spmm_noalloc: scratch memory in a device array built into
the library) against ftc_spmm with a caller workspace: same kernels, so the results must agree bit for
bit, on two calls in a row, the second on a smaller input that leaves most of the buffer's old contents
in place.  Also against the oracle, and the size limit is reported as an error."""
import ctypes as C

import numpy as np
import pytest
import torch

import synth
from parity import TOL, dev_graph, norm_err, quantise
from paper_2412_12218_amd import binding as B

pytestmark = pytest.mark.gpu


def one_call(oracle, g, dtype, D, use_vals, seed):
    rng = np.random.default_rng(seed)
    Xd, X64 = quantise(rng.uniform(-1, 1, size=(g.n, D)).astype(np.float32), dtype)
    vals32 = rng.uniform(-1, 1, size=g.nnz).astype(np.float32) if use_vals else None
    vd = torch.from_numpy(vals32).cuda() if use_vals else None
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    want = B.ftc_spmm(dg, win, vd, Xd)                      # workspace from the caller (torch.empty in the binding)
    got = torch.full((g.n, D), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.ftc_spmm_noalloc(dg, win, vd, Xd, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(got, want), f"{g.name} {dtype} D={D}: differs from ftc_spmm"
    ref, ab = oracle.spmm(g.row_ptr, g.col_idx, None if vals32 is None else vals32.astype(np.float64), X64)
    err = norm_err(got, ref, ab)
    print(f"spmm_noalloc {g.name} n={g.n} nnz={g.nnz} {dtype} D={D}: err {err:.3e}", flush=True)
    assert err < TOL[dtype]


def test_two_calls_in_a_row_the_second_smaller(oracle):
    big = synth.config_graph(5, 1 / 16)         # rows cut by many wave ranges: the carry rows are in use
    small = synth.config_graph(1)
    one_call(oracle, big, torch.float16, 32, True, 1)
    one_call(oracle, small, torch.float16, 32, True, 2)
    one_call(oracle, big, torch.float16, 8, False, 3)       # the narrow-row kernel shares the buffer
    one_call(oracle, small, torch.float32, 16, True, 4)
    one_call(oracle, synth.config_graph(4, 0.02), torch.bfloat16, 64, True, 5)


def test_sizes_beyond_the_buffer_are_refused():
    L = B.lib()
    I = C.c_int32
    n, nnz, D = 1 << 20, 2_000_000_000, 256
    assert L.ftc_spmm_workspace_bytes(n, nnz, D) > (64 << 20)
    g = B.ftc_csr(n, nnz, 0x1000, 0x2000)
    fake = C.c_void_p(0x1000)
    rc = L.ftc_spmm_noalloc(C.byref(g), None, None, fake, I(D), I(1), I(D), C.c_void_p(0x3000), I(D), I(0), None, I(0),
                            I(0), None)
    assert rc == B.FTC_EWORKSPACE
    assert b"built-in buffer" in L.ftc_last_error()
