"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and
rejects bad arguments on the host before anything is launched.  CPU only."""
import ctypes as C
import os
import re

import pytest

from paper_2412_12218_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ftc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ftc_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = declared_symbols()
    assert len(names) >= 15
    for name in names:
        assert hasattr(L, name), name
    assert sorted(B.EXPORTS) == names
    assert L.ftc_version() >= 100


def test_binding_has_same_names():
    for name in declared_symbols():
        if name in ("ftc_last_error",) or name.endswith("_workspace_bytes"):
            continue
        assert callable(getattr(B, name)), name


def _null_call(fn, nargs):
    return fn(*([None] * nargs))


def test_null_graph_is_rejected_on_host():
    L = B.lib()
    z = C.c_size_t(0)
    i = C.c_int32(0)
    assert L.ftc_spmm(None, None, None, None, i, i, i, None, i, i, None, i, i, None, z, None) == B.FTC_EINVAL
    assert b"graph is NULL" in L.ftc_last_error()
    assert L.ftc_build_windows(None, None, None, z, None) == B.FTC_EINVAL
    assert L.ftc_edge_softmax(None, None, None, None, None, z, None) == B.FTC_EINVAL
    assert L.ftc_gcn_norm(None, None, None, None, None) == B.FTC_EINVAL


def test_argument_validation_without_launch():
    L = B.lib()
    fake = C.c_void_p(0x1000)        # never dereferenced: validation fails first
    g = B.ftc_csr(4, 10, 0x1000, 0x2000)
    z = C.c_size_t(0)
    I = C.c_int32
    # negative sizes
    bad = B.ftc_csr(-1, 0, 0x1000, 0)
    assert L.ftc_spmm(C.byref(bad), None, None, fake, I(8), I(1), I(8), fake, I(8), I(0), None, I(0), I(0),
                      None, z, None) == B.FTC_EINVAL
    # unknown dtype
    assert L.ftc_spmm(C.byref(g), None, None, fake, I(8), I(7), I(8), C.c_void_p(0x3000), I(8), I(0), None,
                      I(0), I(0), None, z, None) == B.FTC_EUNSUPPORTED
    # ld < D
    assert L.ftc_spmm(C.byref(g), None, None, fake, I(4), I(1), I(8), C.c_void_p(0x3000), I(8), I(0), None,
                      I(0), I(0), None, z, None) == B.FTC_EINVAL
    # out aliases X
    assert L.ftc_spmm(C.byref(g), None, None, fake, I(8), I(1), I(8), fake, I(8), I(1), None, I(0), I(0),
                      None, z, None) == B.FTC_EINVAL
    # unknown path
    assert L.ftc_spmm(C.byref(g), None, None, fake, I(8), I(1), I(8), C.c_void_p(0x3000), I(8), I(0), None,
                      I(0), I(9), None, z, None) == B.FTC_EINVAL
    # window descriptor inconsistent with n
    w = B.ftc_windows(16, 8, 5, 0x10, 0x20, 0x30, 0x40, 0x50, 0x60)
    assert L.ftc_build_windows(C.byref(g), C.byref(w), fake, C.c_size_t(1 << 30), None) == B.FTC_EINVAL
    w = B.ftc_windows(128, 8, 1, 0x10, 0x20, 0x30, 0x40, 0x50, 0x60)
    assert L.ftc_build_windows(C.byref(g), C.byref(w), fake, C.c_size_t(1 << 30), None) == B.FTC_EUNSUPPORTED
    # workspace too small / missing
    w = B.ftc_windows(16, 8, 1, 0x10, 0x20, 0x30, 0x40, 0x50, 0x60)
    assert L.ftc_build_windows(C.byref(g), C.byref(w), fake, C.c_size_t(8), None) == B.FTC_EWORKSPACE
    assert L.ftc_gcn_layer(C.byref(g), None, None, None, fake, I(8), I(1), I(8), fake, I(8), I(0), fake, I(8), I(0),
                           I(0), None, z, None) == B.FTC_EWORKSPACE
    assert b"workspace" in L.ftc_last_error()
    # gemm arguments: a leading dimension shorter than the row, an output that is the input, no weights
    assert L.ftc_update_gemm(I(4), fake, I(256), I(1), I(512), fake, I(8), C.c_void_p(0x3000), I(8), I(0), None,
                             I(0), None) == B.FTC_EINVAL
    assert L.ftc_update_gemm(I(4), fake, I(512), I(1), I(512), fake, I(8), fake, I(8), I(0), None,
                             I(0), None) == B.FTC_EINVAL
    assert L.ftc_update_gemm(I(4), fake, I(512), I(1), I(512), None, I(8), C.c_void_p(0x3000), I(8), I(0), None,
                             I(0), None) == B.FTC_EINVAL


def test_backward_and_reordering_validate_on_the_host():
    """The backward, reordering and plan entry points refuse bad arguments before anything is launched
    (the fake pointers are never dereferenced)."""
    L = B.lib()
    fake, other = C.c_void_p(0x1000), C.c_void_p(0x3000)
    g = B.ftc_csr(4, 10, 0x1000, 0x2000)
    w = B.ftc_windows(16, 8, 1, 0x10, 0x20, 0x30, 0x40, 0x50, 0x60)
    z, big = C.c_size_t(0), C.c_size_t(1 << 30)
    I, F = C.c_int32, C.c_float
    assert L.ftc_transpose_index(None, None, fake, fake, None) == B.FTC_EINVAL
    assert L.ftc_transpose_index(C.byref(g), None, fake, None, None) == B.FTC_EINVAL                 # flag missing
    assert L.ftc_edge_softmax_backward(C.byref(g), None, None, fake, fake, None, z, None) == B.FTC_EINVAL
    assert L.ftc_edge_softmax_backward(C.byref(g), C.byref(w), fake, fake, fake, None, z, None) == B.FTC_EWORKSPACE
    assert L.ftc_weight_grad(I(8), fake, I(16), I(1), I(16), fake, I(508), I(508), other, fake, big, None) \
        == B.FTC_EUNSUPPORTED                                                                          # too many output columns
    assert L.ftc_weight_grad(I(8), fake, I(16), I(1), I(16), fake, I(8), I(8), other, None, z, None) == B.FTC_EWORKSPACE
    assert L.ftc_gcn_layer_backward(C.byref(g), None, None, None, fake, I(16), I(1), I(16), fake, I(508), None, I(0), I(0),
                                    fake, I(508), other, I(16), other, I(0), fake, big, None) == B.FTC_EUNSUPPORTED
    # H and dY with different leading dimensions
    assert L.ftc_agnn_layer_backward(C.byref(g), None, fake, fake, I(16), I(1), I(16), F(1.0), fake, other, I(24), other,
                                     I(16), I(0), fake, I(0), fake, big, None) == B.FTC_EINVAL
    # the single-pass route needs the window index
    assert L.ftc_agnn_layer_backward_fused(C.byref(g), None, fake, I(16), I(1), I(16), F(1.0), fake, other, I(16), I(0),
                                           other, I(16), C.c_void_p(0x5000), I(16), I(0), fake, None, fake, big, None) == B.FTC_EINVAL
    assert b"window index" in L.ftc_last_error()
    # ... and a width it covers
    assert L.ftc_agnn_layer_backward_fused(C.byref(g), C.byref(w), fake, I(256), I(1), I(256), F(1.0), fake, other, I(256),
                                           I(0), other, I(256), C.c_void_p(0x5000), I(256), I(0), fake, fake, fake, big, None) \
        == B.FTC_EUNSUPPORTED
    assert L.ftc_degree_order(C.byref(g), I(7), fake, fake, fake, big, None) == B.FTC_EINVAL          # unknown ordering
    assert L.ftc_degree_order(C.byref(g), I(0), fake, fake, fake, C.c_size_t(16), None) == B.FTC_EWORKSPACE
    assert L.ftc_permute_graph(C.byref(g), fake, fake, C.c_void_p(0x1000), other, fake, fake, big, None) == B.FTC_EINVAL
    assert b"aliases" in L.ftc_last_error()
    assert L.ftc_label_propagation(C.byref(g), I(-1), fake, fake, big, None) == B.FTC_EINVAL
    assert L.ftc_order_by_key(I(5), None, fake, fake, fake, fake, big, None) == B.FTC_EINVAL
    assert L.ftc_permute_rows(I(5), fake, I(8), I(1), I(8), fake, fake, I(8), None) == B.FTC_EINVAL     # out aliases X
    assert L.ftc_degree_stats(C.byref(g), None, None) == B.FTC_EINVAL
    assert L.ftc_reorder_workspace_bytes(1000, 5000) > 5000 * 4 * 4
    assert L.ftc_agnn_layer_backward_fused_workspace_bytes(1000, 5000, 32) > 1000 * 64 * 4
    assert L.ftc_agnn_layer_backward_fused_workspace_bytes(1000, 5000, 512) == 0


def test_side_streams_are_checked_on_the_host():
    """ftc_build_windows_concurrent: the caller's three streams and four events must be there and distinct; the
    library keeps none of its own (the fake handles are never used: validation fails first)."""
    L = B.lib()
    g = B.ftc_csr(4, 10, 0x1000, 0x2000)
    w = B.ftc_windows(16, 8, 1, 0x10, 0x20, 0x30, 0x40, 0x50, 0x60)
    fake, big = C.c_void_p(0x1000), C.c_size_t(1 << 30)
    side = B.ftc_side_streams()
    assert L.ftc_build_windows_concurrent(C.byref(g), C.byref(w), fake, big, C.byref(side), None) == B.FTC_EINVAL
    assert b"three distinct streams" in L.ftc_last_error()
    for i in range(3):
        side.stream[i], side.join[i] = 0x100 * (i + 1), 0x1000 * (i + 1)
    side.fork = 0x1000                                                   # the same event twice
    assert L.ftc_build_windows_concurrent(C.byref(g), C.byref(w), fake, big, C.byref(side), None) == B.FTC_EINVAL
    side.fork = 0x9000
    assert L.ftc_build_windows_concurrent(C.byref(g), C.byref(w), fake, big, C.byref(side), C.c_void_p(0x200)) \
        == B.FTC_EINVAL                                                  # a side stream that is the caller's stream
    assert L.ftc_build_windows_concurrent(C.byref(g), C.byref(w), None, C.c_size_t(0), C.byref(side), None) \
        == B.FTC_EWORKSPACE


def test_wrong_argument_count_is_rejected_by_the_binding():
    L = B.lib()
    with pytest.raises(TypeError):
        L.ftc_spmm(None, None)
    with pytest.raises(TypeError):
        L.ftc_gcn_layer(None, None, None)


def test_workspace_queries_are_pure_and_monotone():
    L = B.lib()
    a = L.ftc_build_windows_workspace_bytes(1000, 5000, 16, 8)
    b = L.ftc_build_windows_workspace_bytes(2000, 10000, 16, 8)
    assert 0 < a < b
    assert L.ftc_build_windows_workspace_bytes(-1, 0, 16, 8) == 0
    assert L.ftc_gcn_layer_workspace_bytes(1000, 5000, 128, 32) >= 1000 * 32 * 4
    assert L.ftc_agnn_layer_workspace_bytes(1000, 5000, 32) >= 5000 * 4 + 1000 * 4


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libftc.so")
    with pytest.raises(FileNotFoundError):
        B.lib()


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 on its own (no C++ types, no torch, no HIP headers)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_header.c"
    src.write_text('#include "ftc.h"\n'
                   'int main(void) { ftc_csr g; ftc_windows w; ftc_side_streams s; (void)g; (void)w; (void)s;\n'
                   '    return (int)sizeof(ftc_plan) > 0 && FTC_NOALLOC_SCRATCH_MIB > 0 ? 0 : 1; }\n')
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                    "-I", os.path.join(ROOT, "include"), str(src)], check=True)
