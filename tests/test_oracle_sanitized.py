"""The C oracle under the host sanitizers (CPU only): oracle/ftc_oracle.c is compiled together with a small
driver with -fsanitize=address,undefined (both runtimes linked statically, no preloading) and every routine is
run on graphs with empty rows, unsorted and repeated columns, a ragged last window and no entries at all.  The
process must end cleanly, and what it wrote must equal what the ordinary build of the oracle returns: a read or
write beyond an array in the checker would otherwise go unnoticed for as long as the values look right."""
import os
import shutil
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import synth  # noqa: E402
from oracle import ftc_oracle as O  # noqa: E402


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path_factory.mktemp("san") / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-Wall", "-Wextra", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-static-libasan", "-static-libubsan",
           "-o", exe, os.path.join(ROOT, "oracle", "ftc_oracle.c"),
           os.path.join(ROOT, "tests", "sanitize_oracle_driver.c"), "-lm"]
    subprocess.run(cmd, check=True)
    return exe


def _csr(n, rows, cols):
    order = np.argsort(np.asarray(rows), kind="stable")
    rows, cols = np.asarray(rows, dtype=np.int64)[order], np.asarray(cols, dtype=np.int32)[order]
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    np.add.at(row_ptr, rows + 1, 1)
    return np.cumsum(row_ptr).astype(np.int32), cols


def _cases():
    g = synth.rmat(9, 6, 31)                                   # skewed degrees, empty rows, 512 = 32 full windows
    yield "rmat", g.row_ptr, g.col_idx, 24, 7, 16, 8
    g = synth.erdos_renyi(301, 2000, 32)                       # ragged last window (301 = 18 * 16 + 13)
    yield "er", g.row_ptr, g.col_idx, 5, 3, 16, 8
    yield "er_8x16", g.row_ptr, g.col_idx, 5, 3, 8, 16
    rng = np.random.default_rng(33)                            # unsorted rows with repeated columns
    rows = rng.integers(0, 50, 600)
    cols = rng.integers(0, 50, 600)
    rp, ci = _csr(50, rows, cols)
    yield "unsorted_repeats", rp, ci, 9, 4, 16, 8
    yield "no_entries", np.zeros(38, dtype=np.int32), np.zeros(0, dtype=np.int32), 4, 2, 16, 8
    yield "no_nodes", np.zeros(1, dtype=np.int32), np.zeros(0, dtype=np.int32), 4, 2, 16, 8


@pytest.mark.parametrize("case", list(_cases()), ids=lambda c: c[0])
def test_oracle_runs_clean_under_the_sanitizers_and_returns_the_same_values(driver, tmp_path, case):
    name, row_ptr, col_idx, D, d_out, blk_h, blk_w = case
    row_ptr, col_idx = np.ascontiguousarray(row_ptr, dtype=np.int32), np.ascontiguousarray(col_idx, dtype=np.int32)
    n, nnz = row_ptr.size - 1, col_idx.size
    rng = np.random.default_rng(7)
    X = rng.standard_normal((n, D))
    if n > 3:
        X[3] = 0.0                                             # a zero row: the clamped norm
    W = rng.standard_normal((D, d_out))
    beta = 1.7
    fin, fout = str(tmp_path / "case.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        f.write(np.array([n, nnz, D, d_out, blk_h, blk_w], dtype=np.int32).tobytes())
        for a in (row_ptr, col_idx, X, W, np.array([beta])):
            f.write(np.ascontiguousarray(a).tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([driver, fin, fout], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]

    buf = open(fout, "rb").read()
    pos = 0

    def take(count, dtype):
        nonlocal pos
        a = np.frombuffer(buf, dtype=dtype, count=count, offset=pos)
        pos += a.nbytes
        return a

    n_win = (n + blk_h - 1) // blk_h
    vals, dinv = O.gcn_norm(row_ptr, col_idx)
    np.testing.assert_array_equal(take(nnz, np.float64), vals)
    np.testing.assert_array_equal(take(n, np.float64), dinv)
    w = O.build_windows(row_ptr, col_idx, blk_h, blk_w)
    np.testing.assert_array_equal(take(nnz, np.int32), w["edge_to_row"])
    np.testing.assert_array_equal(take(nnz, np.int32), w["edge_to_col"])
    np.testing.assert_array_equal(take(n_win, np.int32), w["block_partition"])
    np.testing.assert_array_equal(take(n_win + 1, np.int32), w["win_col_ptr"])
    np.testing.assert_array_equal(take(nnz, np.int32)[:int(w["summary"][0])], w["win_cols"])
    np.testing.assert_array_equal(take(2, np.int64), w["summary"])
    assert int(take(1, np.int64)[0]) == O.tile_capacity(int(w["summary"][1]), blk_h, blk_w)

    def same(count, want):
        np.testing.assert_allclose(take(count, np.float64), np.asarray(want).ravel(), rtol=1e-14, atol=0)

    y, ya = O.spmm(row_ptr, col_idx, vals, X)
    same(n * D, y), same(n * D, ya)
    rinv = O.row_rnorm(X)
    same(n, rinv)
    s, sa = O.sddmm(row_ptr, col_idx, X, X, rinv, rinv, beta)
    same(nnz, s), same(nnz, sa)
    same(nnz, O.edge_softmax(row_ptr, s))
    Z, Za = O.gemm(X, W)
    same(n * d_out, Z), same(n * d_out, Za)
    gy, ga = O.gcn_layer(row_ptr, col_idx, vals, X, W, relu=True)
    same(n * d_out, gy), same(n * d_out, ga)
    ay, aa, ap = O.agnn_layer(row_ptr, col_idx, X, beta)
    same(n * D, ay), same(n * D, aa), same(nnz, ap)
    assert pos == len(buf)
