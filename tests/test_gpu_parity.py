"""GPU parity: every entry point of libftc, called through the C ABI, against the fp64 CPU
oracle on the same seeded inputs.  Integer outputs bit-exact; float outputs within 2e-3
(16-bit inputs) / 1e-5 (fp32 inputs) of the oracle, normalised by the sum of absolute terms."""
import numpy as np
import pytest
import torch

import synth
from parity import TOL, check_windows, dev_graph, norm_err, quantise, rel_err
from paper_2412_12218_amd import binding as B

pytestmark = pytest.mark.gpu

F32, F16, BF16 = torch.float32, torch.float16, torch.bfloat16
P_TOL = 1e-5     # attention probabilities, relative, whatever the input type (the inputs are exact on both sides)


def say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ graphs used by several tests
def hub_graph():
    """n=700 (not a multiple of 16): one hub row with ~5000 entries incl. duplicates (a window too
    large for LDS), empty rows, unsorted columns."""
    rng = np.random.default_rng(42)
    n = 700
    rows = [rng.integers(0, n, size=rng.integers(0, 12)) for _ in range(n)]
    rows[37] = rng.integers(0, n, size=5000)         # hub with many duplicates
    rows[38] = np.array([], dtype=np.int64)
    rows[699] = rng.integers(0, n, size=300)
    for r in range(100, 140):
        rows[r] = np.array([], dtype=np.int64)       # two fully empty windows
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum([len(r) for r in rows])
    col = np.concatenate(rows).astype(np.int32)
    return synth.Graph(n, row_ptr, col, "hub")


def mixed_density_graph():
    """4096 nodes: windows of the first half draw their columns from a pool of 48 (about ten
    edges per condensed column: matrix-core territory), the second half is Erdos-Renyi sparse."""
    n = 4096
    dense = synth.fill_controlled(n, pool=48, k=30, seed=21)
    sparse = synth.erdos_renyi(n, 4 * n, seed=22)
    rows = []
    for r in range(n):
        src = dense if r < n // 2 else sparse
        rows.append(src.col_idx[src.row_ptr[r]:src.row_ptr[r + 1]])
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum([len(r) for r in rows])
    return synth.Graph(n, row_ptr, np.concatenate(rows).astype(np.int32), "mixed")


@pytest.fixture(scope="module")
def graphs():
    gs = {
        "cfg1": synth.config_graph(1),
        "cfg2s": synth.config_graph(2, 0.2),
        "cfg3s": synth.config_graph(3, 0.1),
        "cfg4s": synth.config_graph(4, 0.03),
        "cfg5s": synth.config_graph(5, 1 / 32),
        "hub": hub_graph(),
        "mixed": mixed_density_graph(),
    }
    return gs


GRAPH_NAMES = ["cfg1", "cfg2s", "cfg3s", "cfg4s", "cfg5s", "hub", "mixed"]


# ------------------------------------------------------------------ validation kernel
def test_validate_csr(graphs):
    g = graphs["cfg1"]
    dg = dev_graph(g)
    assert int(B.ftc_validate_csr(dg).item()) == 0
    bad_col = g.col_idx.copy(); bad_col[5] = g.n
    assert int(B.ftc_validate_csr(B.Graph.from_numpy(g.row_ptr, bad_col)).item()) == 2
    bad_rp = g.row_ptr.copy(); bad_rp[3], bad_rp[4] = bad_rp[4] + 1, bad_rp[3]
    assert int(B.ftc_validate_csr(B.Graph.from_numpy(bad_rp, g.col_idx)).item()) & 1


# ------------------------------------------------------------------ window build (bit-exact)
@pytest.mark.parametrize("name", GRAPH_NAMES)
@pytest.mark.parametrize("blk", [(16, 8), (16, 16), (8, 4), (64, 8), (5, 3)])
def test_build_windows(oracle, graphs, name, blk):
    g = graphs[name]
    if blk != (16, 8) and name in ("cfg2s", "cfg3s", "cfg4s"):
        pytest.skip("other tile shapes are covered on the remaining graphs")
    say(f"build_windows {name} n={g.n} nnz={g.nnz} blk={blk}")
    ref = oracle.build_windows(g.row_ptr, g.col_idx, *blk)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg, *blk)
    torch.cuda.synchronize()
    check_windows(win, ref)
    win2 = B.ftc_build_windows(dg, *blk)     # same answer again (no run-to-run variation)
    check_windows(win2, ref)


def test_build_windows_more_than_one_column_range(oracle):
    """More than 2^20 nodes: large windows take several bitmap passes (one per 2^20 column ids),
    including passes that hold none of a window's columns."""
    rng = np.random.default_rng(77)
    n = (1 << 20) + 70_000
    rows = {}
    rows[5] = rng.integers(0, n, size=3000)                         # both ranges
    rows[6] = rng.integers(0, n, size=2500)
    rows[1_060_000] = rng.integers(1 << 20, n, size=2000)           # upper range only
    rows[500_000] = rng.integers(0, 1 << 20, size=1500)             # lower range only
    rows[500_001] = np.array([n - 1, 0, (1 << 20) - 1, 1 << 20])    # the range borders
    for r in rng.integers(0, n, size=4000):
        rows.setdefault(int(r), rng.integers(0, n, size=rng.integers(1, 40)))
    deg = np.zeros(n, dtype=np.int64)
    for r, c in rows.items():
        deg[r] = len(c)
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(deg)
    col = np.concatenate([rows[r] for r in sorted(rows)]).astype(np.int32)
    g = synth.Graph(n, row_ptr, col)
    ref = oracle.build_windows(g.row_ptr, g.col_idx)
    win = B.ftc_build_windows(dev_graph(g))
    check_windows(win, ref)


def size_class_graph(n, seed):
    """Windows of every size class of the build: a few edges, ~3000 (workgroup, ids in registers),
    ~10000 and ~20000 (workgroup, larger), and hubs of 33000 / 70001 edges (edge-parallel path),
    with duplicates, unsorted columns and a hub in the last, short window."""
    rng = np.random.default_rng(seed)
    deg = rng.integers(0, 9, size=n)
    deg[16 * 3:16 * 4] = 190                  # ~3000 edges in window 3
    deg[16 * 7 + 2] = 10_000                  # one long row
    deg[16 * 9:16 * 10] = 1250                # 20000 edges over 16 rows
    deg[16 * 20:16 * 21] = 2063               # hub: 33008 edges
    deg[16 * 21] = 70_001                     # hub next to it, all in one row
    deg[n - 3:] = 12_000                      # hub in the last window (3 rows when n % 16 == 3)
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(deg)
    col = rng.integers(0, n, size=int(row_ptr[-1])).astype(np.int32)
    lo, hi = row_ptr[16 * 21], row_ptr[16 * 21 + 1]
    col[lo:hi] = rng.integers(0, min(n, 5000), size=hi - lo)     # heavy duplication inside a hub
    return synth.Graph(n, row_ptr, col, "classes")


@pytest.mark.parametrize("n,blk", [(40_003, (16, 8)), (40_003, (64, 8)), (40_003, (5, 3)),
                                   ((1 << 21) + 4099, (16, 8)), ((1 << 22) + 4099, (16, 8))])
def test_build_windows_size_classes(oracle, n, blk):
    """Every size class of the window build, also on a graph with more than 2^21 nodes (three column
    ranges per large window, windows queued in parts) and on one with more than 2^22 nodes (more than four
    ranges: the two-level workgroup kernels and the edge-parallel hub kernels with bitmaps of more than 2^16
    words take the large windows there)."""
    g = size_class_graph(n, seed=n % 1000)
    say(f"build_windows classes n={g.n} nnz={g.nnz} blk={blk}")
    ref = oracle.build_windows(g.row_ptr, g.col_idx, *blk)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg, *blk)
    torch.cuda.synchronize()
    check_windows(win, ref)
    check_windows(B.ftc_build_windows(dg, *blk), ref)


def test_build_windows_degenerate(oracle):
    # no edges at all, and a single node
    for n in (1, 33):
        g = synth.Graph(n, np.zeros(n + 1, dtype=np.int32), np.zeros(0, dtype=np.int32))
        ref = oracle.build_windows(g.row_ptr, g.col_idx)
        win = B.ftc_build_windows(dev_graph(g))
        check_windows(win, ref)
    g = synth.Graph(1, np.array([0, 1], dtype=np.int32), np.array([0], dtype=np.int32))
    check_windows(B.ftc_build_windows(dev_graph(g)), oracle.build_windows(g.row_ptr, g.col_idx))


@pytest.mark.parametrize("which", ["classes", "classes_many_ranges", "cfg5s", "cfg1", "no_edges"])
def test_build_windows_concurrent_on_the_callers_side_streams(oracle, graphs, which):
    """The same index with the independent kernels on three side streams of the caller's: bit-exact against
    the oracle, twice with the same set of streams, and equal to the call that runs in stream order."""
    if which == "classes":
        g = size_class_graph(40_003, seed=3)
    elif which == "classes_many_ranges":   # more than four 2^20-column ranges: the other set of large-window kernels
        g = size_class_graph((1 << 22) + 77, seed=4)
    elif which == "no_edges":
        g = synth.Graph(33, np.zeros(34, dtype=np.int32), np.zeros(0, dtype=np.int32))
    else:
        g = graphs[which]
    ref = oracle.build_windows(g.row_ptr, g.col_idx)
    dg = dev_graph(g)
    side = B.SideStreams()
    for _ in range(2):
        win = B.ftc_build_windows_concurrent(dg, side)
        torch.cuda.synchronize()
        check_windows(win, ref)
    check_windows(B.ftc_build_windows_concurrent(dg, None), ref)
    check_windows(B.ftc_build_windows(dg), ref)


# ------------------------------------------------------------------ GCN normalisation
@pytest.mark.parametrize("name", ["cfg1", "cfg5s", "hub"])
@pytest.mark.parametrize("with_windows", [False, True])
def test_gcn_norm(oracle, graphs, name, with_windows):
    g = graphs[name]
    say(f"gcn_norm {name} windows={with_windows}")
    vals64, dinv64 = oracle.gcn_norm(g.row_ptr, g.col_idx)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg) if with_windows else None
    vals, dinv = B.ftc_gcn_norm(dg, win)
    if name == "hub":   # empty rows: dinv is 0 there and their columns give 0 values; compare the rest
        deg = np.diff(g.row_ptr)
        ok_e = deg[g.col_idx] > 0
        assert rel_err(vals[torch.from_numpy(ok_e).cuda()], vals64[ok_e]) < 1e-6
        assert rel_err(dinv[torch.from_numpy(deg > 0).cuda()], dinv64[deg > 0]) < 1e-6
        assert torch.all(dinv[torch.from_numpy(deg == 0).cuda()] == 0)
    else:
        assert rel_err(vals, vals64) < 1e-6
        assert rel_err(dinv, dinv64) < 1e-6


# ------------------------------------------------------------------ SpMM
def run_spmm(oracle, g, dtype, D, *, use_vals=True, with_windows=True, relu=False, out_dtype=F32,
             pad=0, seed=0, path=B.FTC_PATH_AUTO):
    rng = np.random.default_rng(seed)
    X32 = rng.uniform(-1, 1, size=(g.n, D + pad)).astype(np.float32)
    Xd, X64 = quantise(X32, dtype)
    if pad:
        Xd, X64 = Xd[:, :D], X64[:, :D]
    vals32 = rng.uniform(0.1, 1.0, size=g.nnz).astype(np.float32) * rng.choice([-1.0, 1.0], g.nnz).astype(np.float32)
    ref, ab = oracle.spmm(g.row_ptr, g.col_idx, vals32.astype(np.float64) if use_vals else None, X64)
    if relu:
        ref = np.maximum(ref, 0)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg) if with_windows else None
    vd = torch.from_numpy(vals32).cuda() if use_vals else None
    out = torch.full((g.n, D + pad), 777.0, dtype=out_dtype, device="cuda")[:, :D]
    B.ftc_spmm(dg, win, vd, Xd, out=out, relu=relu, path=path)
    out2 = torch.empty((g.n, D + pad), dtype=out_dtype, device="cuda")[:, :D]    # the same call once more
    B.ftc_spmm(dg, win, vd, Xd, out=out2, relu=relu, path=path)
    torch.cuda.synchronize()
    assert torch.equal(out, out2), "two runs differ"
    return norm_err(out, ref, ab, out_dtype)


@pytest.mark.parametrize("name", GRAPH_NAMES)
@pytest.mark.parametrize("dtype,D", [(F32, 16), (F16, 32), (BF16, 64), (F16, 128), (F16, 16), (F16, 8),
                                     (F32, 4), (F32, 64), (BF16, 8)])
@pytest.mark.parametrize("with_windows", [True, False])
def test_spmm(oracle, graphs, name, dtype, D, with_windows):
    g = graphs[name]
    say(f"spmm {name} {dtype} D={D} windows={with_windows}")
    err = run_spmm(oracle, g, dtype, D, with_windows=with_windows)
    say(f"  err {err:.3e}")
    assert err < TOL[dtype]


@pytest.mark.parametrize("dtype,D,pad", [(F16, 24, 0), (F16, 40, 8), (F32, 12, 4), (F16, 5, 0), (F32, 7, 2),
                                         (BF16, 20, 3), (F16, 64, 64)])
def test_spmm_odd_shapes(oracle, graphs, dtype, D, pad):
    say(f"spmm odd {dtype} D={D} pad={pad}")
    assert run_spmm(oracle, graphs["cfg1"], dtype, D, pad=pad) < TOL[dtype]
    assert run_spmm(oracle, graphs["hub"], dtype, D, pad=pad) < TOL[dtype]


@pytest.mark.parametrize("name", ["cfg1", "cfg5s", "hub"])
@pytest.mark.parametrize("dtype,D,pad", [(F16, 8, 0), (F16, 16, 0), (BF16, 16, 16), (F16, 12, 4), (F16, 6, 2), (F32, 8, 0),
                                         (F32, 6, 2), (F32, 4, 4), (BF16, 2, 6)])
def test_spmm_narrow_rows(oracle, graphs, name, dtype, D, pad):
    """Rows of at most 16 bytes take the lane-per-edge kernel (the wider ones here the four-lane
    layout): with and without edge values, ReLU, 16-bit output, widths below the padded 16 bytes."""
    g = graphs[name]
    say(f"spmm narrow {name} {dtype} D={D} pad={pad}")
    assert run_spmm(oracle, g, dtype, D, pad=pad) < TOL[dtype]
    assert run_spmm(oracle, g, dtype, D, pad=pad, use_vals=False, relu=True) < TOL[dtype]
    assert run_spmm(oracle, g, dtype, D, pad=pad, out_dtype=F16, seed=3) < TOL[dtype]


@pytest.mark.parametrize("out_dtype", [F16, BF16])
def test_spmm_epilogues(oracle, graphs, out_dtype):
    say(f"spmm epilogue {out_dtype}")
    g = graphs["cfg2s"]
    assert run_spmm(oracle, g, F16, 32, relu=True, out_dtype=out_dtype) < 2e-3
    assert run_spmm(oracle, g, F16, 32, use_vals=False) < 2e-3
    assert run_spmm(oracle, g, F32, 16, relu=True) < 1e-5


@pytest.mark.parametrize("name", ["mixed", "cfg1", "cfg5s", "hub", "cfg4s"])
@pytest.mark.parametrize("dtype,D", [(F16, 32), (BF16, 64), (F16, 16), (F16, 8), (F16, 128), (BF16, 24), (F16, 256)])
@pytest.mark.parametrize("path", [B.FTC_PATH_MFMA, B.FTC_PATH_VALU])
def test_spmm_paths(oracle, graphs, name, dtype, D, path):
    """Matrix-core condensed-tile path forced on every eligible window, and the vector path forced
    on every window, against the oracle."""
    g = graphs[name]
    say(f"spmm path={path} {name} {dtype} D={D}")
    err = run_spmm(oracle, g, dtype, D, path=path)
    say(f"  err {err:.3e}")
    assert err < TOL[dtype]
    if name == "mixed":
        assert run_spmm(oracle, g, dtype, D, path=path, relu=True, out_dtype=F16) < TOL[dtype]


@pytest.mark.parametrize("name", ["mixed", "hub", "cfg5s"])
@pytest.mark.parametrize("dtype,D", [(F16, 32), (BF16, 64), (F16, 8), (BF16, 128)])
def test_spmm_mfma_values_of_very_different_size_in_one_tile(oracle, graphs, name, dtype, D):
    """Forced matrix-core path with edge values from 1 down to 2^-60 inside every window, features that are
    exactly zero half of the time (as after a ReLU: an output element may then consist of small terms only)
    and, on `hub`, duplicate entries and unsorted rows.  Every element keeps the bar relative to its own
    terms, and two runs agree bit for bit."""
    g = graphs[name]
    rng = np.random.default_rng(77)
    X32 = rng.uniform(-1, 1, size=(g.n, D)).astype(np.float32)
    X32[rng.random((g.n, D)) < 0.5] = 0.0
    Xd, X64 = quantise(X32, dtype)
    mag = np.exp2(-rng.integers(0, 61, size=g.nnz).astype(np.float64))
    vals32 = (mag * rng.uniform(0.5, 1.0, size=g.nnz) * rng.choice([-1.0, 1.0], g.nnz)).astype(np.float32)
    ref, ab = oracle.spmm(g.row_ptr, g.col_idx, vals32.astype(np.float64), X64)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    vd = torch.from_numpy(vals32).cuda()
    out = B.ftc_spmm(dg, win, vd, Xd, path=B.FTC_PATH_MFMA)
    out2 = B.ftc_spmm(dg, win, vd, Xd, path=B.FTC_PATH_MFMA)
    assert torch.equal(out, out2)
    err = norm_err(out, ref, ab)
    say(f"spmm mfma wide-range values {name} {dtype} D={D} err {err:.3e}")
    assert err < TOL[dtype]


@pytest.mark.parametrize("name", ["mixed", "hub"])
@pytest.mark.parametrize("dtype,D", [(F16, 32), (BF16, 64)])
@pytest.mark.parametrize("beta", [50.0, -50.0, 8.0])
def test_agnn_layer_on_the_matrix_core_path_with_a_large_beta(oracle, graphs, name, dtype, D, beta):
    """The unfused chain with both sparse products forced onto the matrix cores; at |beta| = 50 the
    probabilities of one window span more than forty orders of magnitude."""
    g = graphs[name]
    Hd, H64 = quantise(synth.normal_features(g.n, D, seed=13), dtype)
    ref, ab, pref = oracle.agnn_layer(g.row_ptr, g.col_idx, H64, beta)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    p = torch.empty(g.nnz, dtype=F32, device="cuda")
    out = B.ftc_agnn_layer(dg, win, Hd, beta=beta, edge_p=p, path=B.FTC_PATH_MFMA)
    err = norm_err(out, ref, ab)
    say(f"agnn mfma {name} {dtype} D={D} beta={beta} err {err:.3e}")
    assert err < TOL[dtype]


def test_cfg1_as_written(oracle):
    """The first benchmark configuration literally: the normalised adjacency from the normalisation call goes
    into the aggregation; Erdos-Renyi graph of 2048 nodes, X fp32 2048 x 16 uniform[-1, 1], seed 0; bar 1e-5."""
    g = synth.config_graph(1)
    assert g.n == 2048
    X32 = synth.uniform_features(g.n, 16, seed=0)
    vals64, _ = oracle.gcn_norm(g.row_ptr, g.col_idx)
    ref, ab = oracle.spmm(g.row_ptr, g.col_idx, vals64.astype(np.float32).astype(np.float64), X32.astype(np.float64))
    ref64, _ = oracle.spmm(g.row_ptr, g.col_idx, vals64, X32.astype(np.float64))
    dg = dev_graph(g)
    Xd = torch.from_numpy(X32).cuda()
    for win in (B.ftc_build_windows(dg), None):
        vals, _ = B.ftc_gcn_norm(dg, win)
        out = B.ftc_spmm(dg, win, vals, Xd)
        err = norm_err(out, ref, ab)
        err64 = norm_err(out, ref64, ab)        # against the chain that never rounds the edge values
        say(f"cfg1 as written, windows={win is not None}: err {err:.3e} (unrounded values: {err64:.3e})")
        assert err < 1e-5 and err64 < 1e-5


def test_mfma_path_rejected_where_it_cannot_run(graphs):
    g = graphs["cfg1"]
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    X = torch.zeros((g.n, 16), dtype=F32, device="cuda")
    with pytest.raises(B.FtcError) as ei:
        B.ftc_spmm(dg, win, None, X, path=B.FTC_PATH_MFMA)
    assert ei.value.code == B.FTC_EUNSUPPORTED
    with pytest.raises(B.FtcError) as ei:
        B.ftc_sddmm(dg, win, X, X, path=B.FTC_PATH_MFMA)
    assert ei.value.code == B.FTC_EUNSUPPORTED
    win8 = B.ftc_build_windows(dg, 8, 4)
    Xh = torch.zeros((g.n, 16), dtype=F16, device="cuda")
    with pytest.raises(B.FtcError):
        B.ftc_spmm(dg, win8, None, Xh, path=B.FTC_PATH_MFMA)
    B.ftc_spmm(dg, win8, None, Xh)      # the default path still works with other window heights


def test_forced_paths_on_a_graph_without_entries():
    """No entries: every path clears the output rows (SpMM, AGNN layer) or has nothing to write (SDDMM)."""
    n = 33
    g = synth.Graph(n, np.zeros(n + 1, dtype=np.int32), np.zeros(0, dtype=np.int32), "no_edges")
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    X = torch.randn((n, 32), device="cuda").to(F16)
    for path in (B.FTC_PATH_AUTO, B.FTC_PATH_MFMA, B.FTC_PATH_VALU):
        out = torch.full((n, 32), 5.0, device="cuda")
        B.ftc_spmm(dg, win, None, X, out=out, path=path)
        assert float(out.abs().max()) == 0.0
        assert B.ftc_sddmm(dg, win, X, X, path=path).numel() == 0
        out = torch.full((n, 32), 5.0, device="cuda")
        B.ftc_agnn_layer(dg, win, X, out=out, path=path)
        assert float(out.abs().max()) == 0.0


# ------------------------------------------------------------------ SDDMM
def run_sddmm(oracle, g, dtype, D, *, scales=True, with_windows=True, same=False, seed=1, pad=0,
              path=B.FTC_PATH_AUTO):
    rng = np.random.default_rng(seed)
    Xd, X64 = quantise(rng.standard_normal((g.n, D + pad)).astype(np.float32), dtype)
    if same:
        Yd, Y64 = Xd, X64
    else:
        Yd, Y64 = quantise(rng.standard_normal((g.n, D + pad)).astype(np.float32), dtype)
    if pad:
        Xd, X64, Yd, Y64 = Xd[:, :D], X64[:, :D], Yd[:, :D], Y64[:, :D]
    rs = rng.uniform(0.5, 2.0, g.n).astype(np.float32) if scales else None
    cs = rng.uniform(0.5, 2.0, g.n).astype(np.float32) if scales else None
    alpha = 0.75
    ref, ab = oracle.sddmm(g.row_ptr, g.col_idx, X64, Y64, None if rs is None else rs.astype(np.float64),
                           None if cs is None else cs.astype(np.float64), alpha)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg) if with_windows else None
    rsd = torch.from_numpy(rs).cuda() if scales else None
    csd = torch.from_numpy(cs).cuda() if scales else None
    out = B.ftc_sddmm(dg, win, Xd, Yd, rsd, csd, alpha, path=path)
    out2 = B.ftc_sddmm(dg, win, Xd, Yd, rsd, csd, alpha, path=path)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    return norm_err(out, ref, ab)


@pytest.mark.parametrize("name", GRAPH_NAMES)
@pytest.mark.parametrize("dtype,D", [(F16, 32), (BF16, 64), (F32, 16), (F16, 128), (F16, 8), (F32, 32)])
@pytest.mark.parametrize("with_windows", [True, False])
def test_sddmm(oracle, graphs, name, dtype, D, with_windows):
    g = graphs[name]
    say(f"sddmm {name} {dtype} D={D} windows={with_windows}")
    err = run_sddmm(oracle, g, dtype, D, with_windows=with_windows)
    say(f"  err {err:.3e}")
    assert err < TOL[dtype]


@pytest.mark.parametrize("name", ["mixed", "cfg1", "cfg5s", "hub", "cfg4s"])
@pytest.mark.parametrize("dtype,D", [(F16, 32), (BF16, 64), (F16, 16), (F16, 8), (F16, 128), (BF16, 24), (F16, 256)])
@pytest.mark.parametrize("path", [B.FTC_PATH_MFMA, B.FTC_PATH_VALU, B.FTC_PATH_AUTO])
def test_sddmm_paths(oracle, graphs, name, dtype, D, path):
    g = graphs[name]
    say(f"sddmm path={path} {name} {dtype} D={D}")
    err = run_sddmm(oracle, g, dtype, D, path=path)
    say(f"  err {err:.3e}")
    assert err < TOL[dtype]
    if name == "mixed":
        assert run_sddmm(oracle, g, dtype, D, path=path, scales=False, same=True) < TOL[dtype]


@pytest.mark.parametrize("name", ["cfg1", "cfg5s", "hub", "mixed"])
@pytest.mark.parametrize("dtype,D", [(F16, 32), (BF16, 64), (F32, 16), (F16, 8), (F16, 256), (F16, 5)])
@pytest.mark.parametrize("path", [B.FTC_PATH_AUTO, B.FTC_PATH_MFMA, B.FTC_PATH_VALU])
@pytest.mark.parametrize("same", [True, False])
def test_sddmm_cosine(oracle, graphs, name, dtype, D, path, same):
    """AGNN edge scores alpha * cos(x_i, y_j) without arrays of norms, on every kernel family and
    without a window index; the oracle gets the inverse norms it computes itself.  One row is zero:
    its scores must be exactly 0."""
    g = graphs[name]
    if path == B.FTC_PATH_MFMA and (dtype == F32 or D % 8):
        pytest.skip("matrix-core path needs 16-bit rows of 16-byte pieces")
    rng = np.random.default_rng(41)
    X32 = rng.standard_normal((g.n, D)).astype(np.float32)
    X32[3] = 0
    Xd, X64 = quantise(X32, dtype)
    if same:
        Yd, Y64 = Xd, X64
    else:
        Yd, Y64 = quantise(rng.standard_normal((g.n, D)).astype(np.float32) * 3, dtype)
    ref, ab = oracle.sddmm(g.row_ptr, g.col_idx, X64, Y64, oracle.row_rnorm(X64), oracle.row_rnorm(Y64), -1.5)
    dg = dev_graph(g)
    for win in (B.ftc_build_windows(dg), None):
        out = B.ftc_sddmm(dg, win, Xd, Yd, alpha=-1.5, path=path if win else 0, cosine=True)
        err = norm_err(out, ref, ab)
        say(f"sddmm cosine {name} {dtype} D={D} path={path} same={same} windows={win is not None} err {err:.3e}")
        assert err < TOL[dtype]
        assert float(out.abs().max()) <= 1.5 * (1 + 1e-3)
    with pytest.raises(B.FtcError):
        B.ftc_sddmm(dg, None, Xd, Yd, row_scale=torch.ones(g.n, device="cuda"), cosine=True)


@pytest.mark.parametrize("dtype,D,pad", [(F16, 24, 0), (F16, 5, 0), (F32, 7, 1), (BF16, 40, 8), (F16, 32, 32)])
def test_sddmm_odd_shapes(oracle, graphs, dtype, D, pad):
    say(f"sddmm odd {dtype} D={D} pad={pad}")
    assert run_sddmm(oracle, graphs["cfg1"], dtype, D, pad=pad) < TOL[dtype]
    assert run_sddmm(oracle, graphs["hub"], dtype, D, pad=pad, scales=False, same=True) < TOL[dtype]


# ------------------------------------------------------------------ row norms and edge softmax
@pytest.mark.parametrize("dtype,D", [(F16, 32), (BF16, 64), (F32, 16), (F16, 5)])
def test_row_rnorm(oracle, dtype, D):
    rng = np.random.default_rng(3)
    H32 = rng.standard_normal((1000, D)).astype(np.float32)
    H32[17] = 0
    Hd, H64 = quantise(H32, dtype)
    ref = oracle.row_rnorm(H64)
    got = B.ftc_row_rnorm(Hd)
    assert rel_err(got, ref) < 1e-5 * (1 if dtype == F32 else 10)


@pytest.mark.parametrize("name", GRAPH_NAMES)
@pytest.mark.parametrize("with_windows", [True, False])
def test_edge_softmax(oracle, graphs, name, with_windows):
    g = graphs[name]
    say(f"edge_softmax {name} windows={with_windows}")
    rng = np.random.default_rng(5)
    s32 = (rng.standard_normal(g.nnz) * 2).astype(np.float32)
    ref = oracle.edge_softmax(g.row_ptr, s32.astype(np.float64))
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg) if with_windows else None
    sd = torch.from_numpy(s32).cuda()
    p = B.ftc_edge_softmax(dg, win, sd)
    err = rel_err(p, ref)
    say(f"  err {err:.3e}")
    assert err < 1e-5
    p2 = B.ftc_edge_softmax(dg, win, sd)
    assert torch.equal(p, p2)
    B.ftc_edge_softmax(dg, win, sd, out=sd)           # in place
    assert torch.equal(p, sd)
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    sums = np.bincount(rows, weights=p.cpu().double().numpy(), minlength=g.n)
    assert np.allclose(sums[np.diff(g.row_ptr) > 0], 1.0, atol=1e-5)


@pytest.mark.parametrize("with_windows", [True, False])
def test_edge_softmax_long_rows(oracle, with_windows):
    """Rows of 1, 16, 17, 2048, 2049 and 70000 entries: every length class of the row kernel, and
    rows cut by one, two and many edge ranges of the balanced kernel."""
    lens = [1, 16, 17, 0, 2048, 2049, 70000, 3, 100, 1024, 1024, 5, 1019, 64, 63, 1, 1, 2000]
    row_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    nnz = int(row_ptr[-1])
    g = synth.Graph(len(lens), row_ptr, np.zeros(nnz, dtype=np.int32))
    rng = np.random.default_rng(6)
    s32 = (rng.standard_normal(nnz) * 3 + 50).astype(np.float32)
    ref = oracle.edge_softmax(g.row_ptr, s32.astype(np.float64))
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg) if with_windows else None
    p = B.ftc_edge_softmax(dg, win, torch.from_numpy(s32).cuda())
    assert rel_err(p, ref) < 1e-5


# ------------------------------------------------------------------ update GEMM and layers
@pytest.mark.parametrize("dtype,d_in,d_out", [(F16, 128, 32), (F16, 128, 16), (F16, 16, 8), (BF16, 64, 64),
                                              (F32, 16, 8), (F16, 32, 8), (F16, 20, 5), (F32, 256, 64)])
@pytest.mark.parametrize("relu", [False, True])
def test_update_gemm(oracle, dtype, d_in, d_out, relu):
    say(f"gemm {dtype} {d_in}x{d_out} relu={relu}")
    n = 3000 + 37
    Xd, X64 = quantise(synth.uniform_features(n, d_in, seed=7), dtype)
    Wd, W64 = quantise(synth.glorot_uniform(d_in, d_out, seed=8), dtype)
    ref, ab = oracle.gemm(X64, W64)
    if relu:
        ref = np.maximum(ref, 0)
    Z = B.ftc_update_gemm(Xd, Wd, relu=relu)
    assert norm_err(Z, ref, ab) < TOL[dtype]
    Zh = B.ftc_update_gemm(Xd, Wd, relu=relu, out_dtype=F16)
    assert norm_err(Zh, ref, ab, F16) < TOL[dtype]


@pytest.mark.parametrize("dtype,d_in,d_out", [(F16, 1432, 16), (F16, 3704, 7), (BF16, 264, 64), (F16, 128, 100),
                                              (BF16, 520, 130), (F32, 1000, 16), (F32, 300, 70), (F32, 4100, 5),
                                              (F16, 1433, 16), (F32, 3703, 6), (BF16, 257, 65)])
def test_update_gemm_wide_shapes(oracle, dtype, d_in, d_out):
    """Beyond the shapes that keep W on chip: the contraction dimension in chunks, more than 64 output
    columns in groups (feature matrices of citation graphs have 1433 and 3703 columns); odd widths take
    the element-wise kernel.  A ragged last row tile, ReLU, row scales and a 16-bit output ride along."""
    say(f"gemm wide {dtype} {d_in}x{d_out}")
    n = 1000 + 21
    Xd, X64 = quantise(synth.uniform_features(n, d_in, seed=7), dtype)
    Wd, W64 = quantise(synth.glorot_uniform(d_in, d_out, seed=8), dtype)
    ref, ab = oracle.gemm(X64, W64)
    Z = B.ftc_update_gemm(Xd, Wd)
    assert norm_err(Z, ref, ab) < TOL[dtype]
    sc32 = np.random.default_rng(5).uniform(-2, 2, size=n).astype(np.float32)
    ref2 = np.maximum(ref * sc32.astype(np.float64)[:, None], 0)
    Zh = B.ftc_update_gemm(Xd, Wd, relu=True, row_scale=torch.from_numpy(sc32).cuda(), out_dtype=F16)
    assert norm_err(Zh, ref2, ab * np.abs(sc32.astype(np.float64))[:, None], F16) < TOL[dtype]


@pytest.mark.parametrize("dtype,d_in,d_out,pad", [(F16, 1433, 16, 7), (BF16, 100, 24, 4), (F16, 3703, 6, 1),
                                                  (F16, 9, 3, 7), (BF16, 250, 70, 6)])
def test_update_gemm_odd_width_in_padded_rows(oracle, dtype, d_in, d_out, pad):
    """A width that is no multiple of 8 stored in 16-byte aligned rows: the matrix cores still take it, and
    the padding of the rows (NaN here) never reaches the result."""
    n = 777
    X32 = synth.uniform_features(n, d_in + pad, seed=3)
    X32[:, d_in:] = np.nan
    Xd, X64 = quantise(X32, dtype)
    Xd, X64 = Xd[:, :d_in], X64[:, :d_in]
    Wd, W64 = quantise(synth.glorot_uniform(d_in, d_out, seed=4), dtype)
    ref, ab = oracle.gemm(X64, W64)
    Z = B.ftc_update_gemm(Xd, Wd)
    assert norm_err(Z, ref, ab) < TOL[dtype]


def test_gcn_layer_with_a_wide_input(oracle, graphs):
    """First layer of a GCN on a feature matrix wider than the on-chip shapes (d_in = 1432 -> 16)."""
    g = graphs["cfg1"]
    vals64, _ = oracle.gcn_norm(g.row_ptr, g.col_idx)
    vals32 = vals64.astype(np.float32)
    Xd, X64 = quantise(synth.uniform_features(g.n, 1432, seed=9), F16)
    Wd, W64 = quantise(synth.glorot_uniform(1432, 16, seed=10), F16)
    ref, ab = oracle.gcn_layer(g.row_ptr, g.col_idx, vals32.astype(np.float64), X64, W64, relu=True)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    out = B.ftc_gcn_layer(dg, win, torch.from_numpy(vals32).cuda(), Xd, Wd, relu=True)
    err = norm_err(out, ref, ab)
    say(f"gcn_layer wide input err {err:.3e}")
    assert err < TOL[F16]


@pytest.mark.parametrize("name,dtype,d_in,d_out", [("cfg1", F32, 16, 16), ("cfg2s", F16, 128, 32),
                                                   ("cfg5s", F16, 128, 16), ("cfg5s", F16, 16, 8),
                                                   ("hub", BF16, 64, 24)])
@pytest.mark.parametrize("relu", [False, True])
def test_gcn_layer(oracle, graphs, name, dtype, d_in, d_out, relu):
    g = graphs[name]
    say(f"gcn_layer {name} {dtype} {d_in}->{d_out} relu={relu}")
    vals64, _ = oracle.gcn_norm(g.row_ptr, g.col_idx)
    vals32 = np.nan_to_num(vals64, posinf=0.0).astype(np.float32)   # hub graph has empty rows
    Xd, X64 = quantise(synth.uniform_features(g.n, d_in, seed=9), dtype)
    Wd, W64 = quantise(synth.glorot_uniform(d_in, d_out, seed=10), dtype)
    ref, ab = oracle.gcn_layer(g.row_ptr, g.col_idx, vals32.astype(np.float64), X64, W64, relu=relu)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    out = B.ftc_gcn_layer(dg, win, torch.from_numpy(vals32).cuda(), Xd, Wd, relu=relu)
    err = norm_err(out, ref, ab)
    say(f"  err {err:.3e}")
    assert err < TOL[dtype]


@pytest.mark.parametrize("name,dtype,d_in,d_out", [("cfg1", F32, 16, 16), ("cfg2s", F16, 128, 32),
                                                   ("cfg5s", F16, 128, 16), ("cfg5s", F16, 16, 8),
                                                   ("hub", BF16, 64, 24), ("mixed", F16, 32, 64)])
@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("path", [B.FTC_PATH_AUTO, B.FTC_PATH_MFMA])
def test_gcn_layer_factored(oracle, graphs, name, dtype, d_in, d_out, relu, path):
    """Factored normalisation: the layer gets dinv instead of per-edge values; the oracle gets the
    products dinv[i] * dinv[j] of the same fp32 numbers."""
    g = graphs[name]
    if path == B.FTC_PATH_MFMA and dtype != F16:
        pytest.skip("the intermediate X*W is fp32 for these inputs; the matrix-core path is 16-bit only")
    say(f"gcn_layer factored {name} {dtype} {d_in}->{d_out} relu={relu} path={path}")
    _, dinv64 = oracle.gcn_norm(g.row_ptr, g.col_idx)
    dinv32 = np.nan_to_num(dinv64, posinf=0.0).astype(np.float32)
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    vals64 = dinv32[rows].astype(np.float64) * dinv32[g.col_idx].astype(np.float64)
    Xd, X64 = quantise(synth.uniform_features(g.n, d_in, seed=9), dtype)
    Wd, W64 = quantise(synth.glorot_uniform(d_in, d_out, seed=10), dtype)
    ref, ab = oracle.gcn_layer(g.row_ptr, g.col_idx, vals64, X64, W64, relu=relu)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    out = B.ftc_gcn_layer(dg, win, None, Xd, Wd, relu=relu, dinv=torch.from_numpy(dinv32).cuda(), path=path)
    err = norm_err(out, ref, ab)
    say(f"  err {err:.3e}")
    assert err < TOL[dtype]
    out_nw = B.ftc_gcn_layer(dg, None, None, Xd, Wd, relu=relu, dinv=torch.from_numpy(dinv32).cuda())
    assert norm_err(out_nw, ref, ab) < TOL[dtype]


@pytest.mark.parametrize("name", ["cfg1", "hub", "mixed"])
@pytest.mark.parametrize("dtype,D", [(F16, 32), (F32, 16), (BF16, 24), (F16, 5)])
@pytest.mark.parametrize("path", [B.FTC_PATH_AUTO, B.FTC_PATH_MFMA, B.FTC_PATH_VALU])
def test_spmm_out_scale(oracle, graphs, name, dtype, D, path):
    """out_scale multiplies output row i before the ReLU (negative factors flip what survives)."""
    g = graphs[name]
    if path == B.FTC_PATH_MFMA and (dtype == F32 or D % 8):
        pytest.skip("matrix-core path needs 16-bit rows of 16-byte pieces")
    rng = np.random.default_rng(31)
    Xd, X64 = quantise(rng.uniform(-1, 1, size=(g.n, D)).astype(np.float32), dtype)
    vals32 = rng.uniform(-1, 1, size=g.nnz).astype(np.float32)
    sc32 = rng.uniform(-2, 2, size=g.n).astype(np.float32)
    ref, ab = oracle.spmm(g.row_ptr, g.col_idx, vals32.astype(np.float64), X64)
    ref = np.maximum(ref * sc32.astype(np.float64)[:, None], 0)
    ab = ab * np.abs(sc32.astype(np.float64))[:, None]
    dg = dev_graph(g)
    for win in (B.ftc_build_windows(dg), None):
        out = B.ftc_spmm(dg, win, torch.from_numpy(vals32).cuda(), Xd, relu=True, path=path if win else 0,
                         out_scale=torch.from_numpy(sc32).cuda())
        assert norm_err(out, ref, ab) < TOL[dtype]


@pytest.mark.parametrize("dtype,d_in,d_out", [(F16, 128, 16), (BF16, 64, 64), (F32, 16, 8), (F16, 20, 5)])
def test_update_gemm_row_scale(oracle, dtype, d_in, d_out):
    n = 2000 + 5
    Xd, X64 = quantise(synth.uniform_features(n, d_in, seed=7), dtype)
    Wd, W64 = quantise(synth.glorot_uniform(d_in, d_out, seed=8), dtype)
    sc32 = np.random.default_rng(32).uniform(-2, 2, size=n).astype(np.float32)
    ref, ab = oracle.gemm(X64, W64)
    ref = np.maximum(ref * sc32.astype(np.float64)[:, None], 0)
    ab = ab * np.abs(sc32.astype(np.float64))[:, None]
    Z = B.ftc_update_gemm(Xd, Wd, relu=True, row_scale=torch.from_numpy(sc32).cuda())
    assert norm_err(Z, ref, ab) < TOL[dtype]


@pytest.mark.parametrize("name,dtype,D", [("cfg1", F32, 16), ("cfg3s", F16, 32), ("cfg5s", F16, 32),
                                          ("cfg4s", BF16, 64), ("hub", F16, 8), ("hub", F16, 128),
                                          ("mixed", BF16, 16), ("cfg5s", F32, 32), ("hub", F16, 24)])
@pytest.mark.parametrize("beta", [1.0, 2.5, -3.0])
def test_agnn_layer(oracle, graphs, name, dtype, D, beta):
    """Both routes of the layer: the unfused chain (taken when the probabilities are requested) and
    the single-pass fused kernel, each against the oracle."""
    g = graphs[name]
    say(f"agnn_layer {name} {dtype} D={D} beta={beta}")
    Hd, H64 = quantise(synth.normal_features(g.n, D, seed=11), dtype)
    ref, ab, pref = oracle.agnn_layer(g.row_ptr, g.col_idx, H64, beta)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    p = torch.empty(g.nnz, dtype=F32, device="cuda")
    out = B.ftc_agnn_layer(dg, win, Hd, beta=beta, edge_p=p)
    err = norm_err(out, ref, ab)
    perr = rel_err(p, pref)
    say(f"  unfused err {err:.3e} p err {perr:.3e}")
    assert err < TOL[dtype]
    assert perr < P_TOL
    out2 = B.ftc_agnn_layer(dg, win, Hd, beta=beta)      # fused: no P output
    err2 = norm_err(out2, ref, ab)
    say(f"  fused err {err2:.3e}")
    assert err2 < TOL[dtype]
    out3 = B.ftc_agnn_layer(dg, win, Hd, beta=beta)
    assert torch.equal(out2, out3)
    out4 = B.ftc_agnn_layer(dg, None, Hd, beta=beta)     # no window index: row kernels
    assert norm_err(out4, ref, ab) < TOL[dtype]


def test_agnn_layer_beyond_the_single_pass_beta_range(oracle, graphs):
    """|beta| >= 43: exp(-2 |beta|) is no fp32 number any more; the layer takes the chain with the
    row-wise softmax, and the outputs only the single pass can give are refused."""
    g = graphs["cfg1"]
    Hd, H64 = quantise(synth.normal_features(g.n, 32, seed=12), F16)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    for beta in (60.0, -75.0):
        ref, ab, _ = oracle.agnn_layer(g.row_ptr, g.col_idx, H64, beta)
        out = B.ftc_agnn_layer(dg, win, Hd, beta=beta)
        assert torch.all(torch.isfinite(out))
        assert norm_err(out, ref, ab) < 2e-3
    with pytest.raises(B.FtcError):
        B.ftc_agnn_layer(dg, win, Hd, beta=60.0, row_z=torch.empty(g.n, dtype=F32, device="cuda"))
    z = torch.ones(g.n, dtype=F32, device="cuda")
    with pytest.raises(B.FtcError):
        B.ftc_agnn_layer_backward_fused(dg, win, Hd, z, Hd.float(), Hd.clone(), beta=60.0)


def test_agnn_layer_fused_large_beta_and_fp16_out(oracle, graphs):
    g = graphs["cfg5s"]
    Hd, H64 = quantise(synth.normal_features(g.n, 32, seed=12), F16)
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    for beta in (20.0, -20.0, 0.0):
        ref, ab, _ = oracle.agnn_layer(g.row_ptr, g.col_idx, H64, beta)
        out = B.ftc_agnn_layer(dg, win, Hd, beta=beta, out_dtype=F16)
        err = norm_err(out, ref, ab, F16)
        say(f"agnn fused beta={beta} err {err:.3e}")
        assert err < 2e-3


# ------------------------------------------------------------------ the step as a HIP graph
def test_hot_path_step_replayed_as_a_graph_matches_eager_runs():
    """Capture the whole step (window build with its side streams, both models) once, replay it several
    times with eager work and synchronisations in between, and compare every replay with the eager
    result bit for bit (the kernels are reproducible); the outputs are poisoned before each replay."""
    from paper_2412_12218_amd.models import HotPath
    g = synth.config_graph(5, 1 / 32)
    dg = dev_graph(g)
    hp = HotPath(dg)
    h16 = lambda a: torch.from_numpy(a).to(F16).cuda()
    X = h16(synth.normal_features(g.n, 128, 1))
    W1, W2 = h16(synth.glorot_uniform(128, 16, 2)), h16(synth.glorot_uniform(16, 8, 3))
    Win, Wout = h16(synth.glorot_uniform(128, 32, 4)), h16(synth.glorot_uniform(32, 8, 5))
    betas = [1.0, 0.5, -1.0, 2.0]
    hp.step(X, W1, W2, Win, Wout, betas)
    torch.cuda.synchronize()
    keep = [t.clone() for t in (hp.gcn_out, hp.agnn_out, hp.win.edge_to_col, hp.win.win_cols, hp.win.summary, hp.dinv)]
    # a second object whose FIRST use is the capture: the library keeps no state that an eager call would have
    # to create beforehand (the side streams of the window build are the caller's)
    hp = HotPath(dg)
    graph = hp.capture(X, W1, W2, Win, Wout, betas)
    for rep in range(4):
        for t in (hp.gcn_out, hp.agnn_out, hp.dinv):
            t.fill_(float("nan"))
        hp.win.edge_to_col.fill_(-7)
        hp.win.summary.zero_()
        scratch = torch.randn(1 << 20, device="cuda").sum()          # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        now = (hp.gcn_out, hp.agnn_out, hp.win.edge_to_col, hp.win.win_cols, hp.win.summary, hp.dinv)
        n_cols = int(hp.win.summary[0].item())
        for a, b in zip(keep, now):
            if a is keep[3]:
                assert torch.equal(a[:n_cols], b[:n_cols]), f"replay {rep}"
            else:
                assert torch.equal(a, b), f"replay {rep}"
        del scratch
    hp.step(X, W1, W2, Win, Wout, betas)                              # and eager calls still work afterwards
    torch.cuda.synchronize()
    assert torch.equal(hp.agnn_out, keep[1])


# ------------------------------------------------------------------ seeded sweep over shapes
def random_graph(rng, n):
    """Random degrees with empty rows, a few long rows (several wave ranges) and duplicates."""
    deg = rng.integers(0, 12, size=n)
    deg[rng.random(n) < 0.2] = 0
    # (long rows only where the columns are spread: a thousand copies of the same term make fp32
    # summation drift by a rounding error per term, beyond the 1e-5 bar, whatever the order)
    for _ in range(rng.integers(0, 3) if n >= 500 else 0):
        deg[rng.integers(0, n)] = rng.integers(600, 2600)
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(deg)
    col = rng.integers(0, n, size=int(row_ptr[-1])).astype(np.int32)
    return synth.Graph(n, row_ptr, col, "random")


@pytest.mark.parametrize("case", range(24))
def test_spmm_sddmm_agnn_random_shapes(oracle, case):
    """Seeded sweep: node counts from 1 to a few thousand, every feature width from 1 to 40 with the
    padding that makes rows 16-byte aligned or not, all three element types, with and without edge
    values: SpMM (whichever kernel the shape selects), cosine SDDMM and the AGNN layer."""
    rng = np.random.default_rng(1000 + case)
    n = int(rng.choice([1, 2, 15, 16, 17, 63, 500, 1025, 3000]))
    g = random_graph(rng, n)
    dtype = [F32, F16, BF16][case % 3]
    D = int(rng.integers(1, 41))
    pad = int(rng.choice([0, (-D) % 8, (-D) % 4, 3]))
    say(f"random case {case}: n={n} nnz={g.nnz} {dtype} D={D} pad={pad}")
    assert run_spmm(oracle, g, dtype, D, pad=pad, use_vals=bool(case & 1), relu=bool(case & 2), seed=case) < TOL[dtype]
    if g.nnz == 0:
        return
    Hd, H64 = quantise(synth.normal_features(n, D + pad, seed=case), dtype)
    Hd, H64 = Hd[:, :D], H64[:, :D]
    dg = dev_graph(g)
    win = B.ftc_build_windows(dg)
    ref, ab, _ = oracle.agnn_layer(g.row_ptr, g.col_idx, H64, 1.5)
    out = B.ftc_agnn_layer(dg, win, Hd, beta=1.5)
    assert norm_err(out, ref, ab) < TOL[dtype]
    Hn = H64 / np.maximum(np.sqrt((H64 * H64).sum(axis=1)), 1e-12)[:, None]
    sref, sab = oracle.sddmm(g.row_ptr, g.col_idx, Hn, Hn)
    s = B.ftc_sddmm(dg, win, Hd, Hd, cosine=True)
    serr = norm_err(s, sref, sab)
    say(f"  cosine sddmm err {serr:.3e}")
    assert serr < TOL[dtype]


def test_spmm_narrow_rows_at_slot_and_wave_boundaries(oracle):
    """Row lengths that end exactly on slot (16 edges) and wave (512 / 1024 edges) boundaries, a row
    covering several whole waves, empty rows in between, and a total that is a multiple of 1024."""
    deg = [16, 0, 16, 32, 0, 0, 1024, 1, 15, 512, 3000, 0, 48, 1024 - 16, 2048, 0, 7]
    deg.append((-sum(deg)) % 1024 + 1024)
    n = len(deg)
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(deg)
    assert row_ptr[-1] % 1024 == 0
    rng = np.random.default_rng(5)
    g = synth.Graph(n, row_ptr, rng.integers(0, n, size=int(row_ptr[-1])).astype(np.int32), "boundaries")
    for dtype, D in ((F16, 8), (F16, 16), (F32, 4), (F32, 8), (BF16, 5)):
        pad = (-D) % (4 if dtype == F32 else 8)
        say(f"boundaries {dtype} D={D}")
        e1 = run_spmm(oracle, g, dtype, D, pad=pad)
        e2 = run_spmm(oracle, g, dtype, D, pad=pad, use_vals=False)
        say(f"  err {e1:.3e} {e2:.3e}")
        assert e1 < TOL[dtype] and e2 < TOL[dtype]
