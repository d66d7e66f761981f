"""Pins of the fp64 CPU oracle against things other than itself: hand-worked examples,
dense brute force (numpy dense algebra on tiny graphs), closed forms and invariants.
CPU only."""
import numpy as np
import pytest
import scipy.sparse as sp

import synth
from conftest import golden_lines


def dense_adj(g, vals=None):
    """Dense matrix built entry by entry; duplicates add up."""
    A = np.zeros((g.n, g.n))
    for i in range(g.n):
        for e in range(g.row_ptr[i], g.row_ptr[i + 1]):
            A[i, g.col_idx[e]] += 1.0 if vals is None else vals[e]
    return A


def small_graphs():
    out = [synth.erdos_renyi(48, 120, seed=11), synth.erdos_renyi(64, 40, seed=12, self_loops=False),
           synth.chung_lu(64, 2.2, 6, seed=13), synth.rmat(6, 4, seed=14),
           synth.sbm(4, 12, 150, 30, seed=15)]
    return out


PATH_RP = np.array([0, 2, 5, 8, 10], dtype=np.int32)
PATH_CI = np.array([0, 1, 0, 1, 2, 1, 2, 3, 2, 3], dtype=np.int32)


# ---------------------------------------------------------------- input generator (CSR build)
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_csr_build_matches_dense_bruteforce(seed):
    rng = np.random.default_rng(seed)
    n, m = 40, 150
    u, v = rng.integers(0, n, m), rng.integers(0, n, m)
    g = synth.csr_from_pairs(n, u, v, self_loops=True)
    D = np.zeros((n, n), dtype=bool)
    for a, b in zip(u, v):
        if a != b:
            D[a, b] = D[b, a] = True
    D[np.arange(n), np.arange(n)] = True
    A = dense_adj(g)
    assert np.array_equal(A > 0, D)
    assert A.max() == 1.0                       # deduplicated
    assert np.array_equal(A, A.T)
    for i in range(n):                          # ascending columns
        c = g.col_idx[g.row_ptr[i]:g.row_ptr[i + 1]]
        assert np.all(np.diff(c) > 0)
    pairs = {(min(a, b), max(a, b)) for a, b in zip(u, v) if a != b}
    assert g.nnz == 2 * len(pairs) + n


# ---------------------------------------------------------------- GCN normalisation
def test_gcn_norm_hand_path(oracle):
    L = golden_lines("h1_gcn_path4.txt")
    vals, dinv = oracle.gcn_norm(PATH_RP, PATH_CI)
    X = np.array([[1, -1], [2, 0], [3, 1], [4, 2.0]])
    want = np.array([[float(t) for t in ln.split()] for ln in L[:4]])
    got, _ = oracle.spmm(PATH_RP, PATH_CI, vals, X)
    assert np.allclose(got, want, atol=2e-6)
    ones, _ = oracle.spmm(PATH_RP, PATH_CI, vals, np.ones((4, 1)))
    assert np.allclose(ones[:, 0], [float(t) for t in L[4].split()], atol=2e-6)
    d = np.array([2, 3, 3, 2.0])
    sq, _ = oracle.spmm(PATH_RP, PATH_CI, vals, np.sqrt(d)[:, None])
    assert np.allclose(sq[:, 0], [float(t) for t in L[5].split()], atol=2e-6)
    assert np.allclose(dinv, 1 / np.sqrt(d), rtol=1e-15)


def test_gcn_norm_hand_star(oracle):
    L = golden_lines("h1_gcn_star4.txt")
    g = synth.csr_from_pairs(4, [0, 0, 0], [1, 2, 3])
    vals, _ = oracle.gcn_norm(g.row_ptr, g.col_idx)
    ones, _ = oracle.spmm(g.row_ptr, g.col_idx, vals, np.ones((4, 1)))
    assert np.allclose(ones[:, 0], [float(t) for t in L[0].split()], atol=2e-6)
    A = dense_adj(g, vals)
    assert abs(A[0, 0] - 0.25) < 1e-15 and abs(A[1, 1] - 0.5) < 1e-15
    assert abs(A[0, 2] - 1 / np.sqrt(8)) < 1e-15


@pytest.mark.parametrize("gi", range(5))
def test_gcn_norm_closed_forms(oracle, gi):
    g = small_graphs()[gi]
    if gi == 1:  # that graph has no self-loops and may have empty rows: rebuild with loops
        g = synth.erdos_renyi(64, 40, seed=12, self_loops=True)
    vals, dinv = oracle.gcn_norm(g.row_ptr, g.col_idx)
    deg = np.diff(g.row_ptr).astype(np.float64)
    A = dense_adj(g, vals)
    # symmetric, and equal to D^-1/2 (A+I) D^-1/2 assembled with dense algebra
    P = dense_adj(g)
    want = np.diag(deg ** -0.5) @ P @ np.diag(deg ** -0.5)
    assert np.allclose(A, want, rtol=1e-14, atol=0)
    assert np.allclose(A, A.T, rtol=1e-15)
    # sqrt(d~) is an eigenvector with eigenvalue 1
    out, _ = oracle.spmm(g.row_ptr, g.col_idx, vals, np.sqrt(deg)[:, None])
    assert np.allclose(out[:, 0], np.sqrt(deg), rtol=1e-13)
    # (A^ 1)_i = d_i^-1/2 * sum_j d_j^-1/2 over stored neighbours
    ones, _ = oracle.spmm(g.row_ptr, g.col_idx, vals, np.ones((g.n, 1)))
    want1 = np.array([deg[i] ** -0.5 * sum(deg[j] ** -0.5 for j in g.col_idx[g.row_ptr[i]:g.row_ptr[i + 1]])
                      for i in range(g.n)])
    assert np.allclose(ones[:, 0], want1, rtol=1e-13)


def test_gcn_norm_regular_graph_rowsum_one(oracle):
    n = 30  # ring: every node has two neighbours + itself
    g = synth.csr_from_pairs(n, np.arange(n), (np.arange(n) + 1) % n)
    vals, _ = oracle.gcn_norm(g.row_ptr, g.col_idx)
    ones, _ = oracle.spmm(g.row_ptr, g.col_idx, vals, np.ones((n, 3)))
    assert np.allclose(ones, 1.0, rtol=1e-15)


# ---------------------------------------------------------------- window build
def parse_h3():
    L = golden_lines("h3_windows.txt")
    cases = []
    for k in range(0, len(L), 11):
        ints = [np.array([int(t) for t in ln.split()], dtype=np.int64) for ln in L[k + 1:k + 11]]
        cases.append((L[k], ints))
    return cases


@pytest.mark.parametrize("case", parse_h3(), ids=lambda c: c[0])
def test_windows_hand_examples(oracle, case):
    _, (n, blk, rp, ci, e2r, e2c, bp, wcp, wc, summ) = case
    w = oracle.build_windows(rp, ci, int(blk[0]), int(blk[1]))
    assert int(n[0]) == rp.size - 1
    assert np.array_equal(w["edge_to_row"], e2r)
    assert np.array_equal(w["edge_to_col"], e2c)
    assert np.array_equal(w["block_partition"], bp)
    assert np.array_equal(w["win_col_ptr"], wcp)
    assert np.array_equal(w["win_cols"], wc)
    assert np.array_equal(w["summary"], summ)


def windows_bruteforce(g, blk_h, blk_w):
    """Python sets and list.index: nothing in common with the C routine."""
    n_win = (g.n + blk_h - 1) // blk_h
    e2r = np.zeros(g.nnz, dtype=np.int64)
    e2c = np.zeros(g.nnz, dtype=np.int64)
    wc, wcp, bp = [], [0], []
    for w in range(n_win):
        rows = range(w * blk_h, min(g.n, (w + 1) * blk_h))
        S = sorted({int(g.col_idx[e]) for r in rows for e in range(g.row_ptr[r], g.row_ptr[r + 1])})
        for r in rows:
            for e in range(g.row_ptr[r], g.row_ptr[r + 1]):
                e2r[e] = r
                e2c[e] = S.index(int(g.col_idx[e]))
        wc += S
        wcp.append(len(wc))
        bp.append(-(-len(S) // blk_w))
    return e2r, e2c, np.array(bp), np.array(wcp), np.array(wc)


@pytest.mark.parametrize("gi", range(5))
@pytest.mark.parametrize("blk", [(16, 8), (4, 2), (5, 3), (16, 16)])
def test_windows_bruteforce_and_invariants(oracle, gi, blk):
    g = small_graphs()[gi]
    w = oracle.build_windows(g.row_ptr, g.col_idx, *blk)
    e2r, e2c, bp, wcp, wc = windows_bruteforce(g, *blk)
    assert np.array_equal(w["edge_to_row"], e2r)
    assert np.array_equal(w["edge_to_col"], e2c)
    assert np.array_equal(w["block_partition"], bp)
    assert np.array_equal(w["win_col_ptr"], wcp)
    assert np.array_equal(w["win_cols"], wc)
    assert w["summary"][0] == len(wc) <= g.nnz
    assert w["summary"][1] == bp.sum()
    # invariants
    win_of_edge = w["edge_to_row"] // blk[0]
    assert np.array_equal(w["win_cols"][w["win_col_ptr"][win_of_edge] + w["edge_to_col"]], g.col_idx)
    for k in range(w["n_windows"]):
        S = w["win_cols"][w["win_col_ptr"][k]:w["win_col_ptr"][k + 1]]
        assert np.all(np.diff(S) > 0)
    assert np.all(g.row_ptr[w["edge_to_row"]] <= np.arange(g.nnz))
    assert np.all(np.arange(g.nnz) < g.row_ptr[w["edge_to_row"] + 1])


def test_windows_unsorted_and_duplicate_columns(oracle):
    # rows 0:{7,3,7}  1:{3,9}  2:{}  3:{1}; duplicates keep their own edge, share a column
    rp = np.array([0, 3, 5, 5, 6]); ci = np.array([7, 3, 7, 3, 9, 1])
    w = oracle.build_windows(rp, ci, 4, 2)
    assert list(w["win_cols"]) == [1, 3, 7, 9]
    assert list(w["edge_to_col"]) == [2, 1, 2, 1, 3, 0]
    assert list(w["edge_to_row"]) == [0, 0, 0, 1, 1, 3]
    assert list(w["block_partition"]) == [2]


def test_tile_capacity_matches_paper_table(oracle):
    for ln in golden_lines("paper_dataset_table.txt"):
        _, blocks, edges = ln.split()
        assert oracle.tile_capacity(int(blocks), 16, 8) == int(edges)


def test_windows_capacity_scatter_roundtrip(oracle):
    """Scatter every edge into its (window, block, row-in-window, column-in-block) cell of the
    padded tile array and read the adjacency back; checks the capacity identity too."""
    g = small_graphs()[0]
    H, W = 16, 8
    w = oracle.build_windows(g.row_ptr, g.col_idx, H, W)
    cap = oracle.tile_capacity(w["summary"][1], H, W)
    tiles = np.zeros(cap)
    blk_base = np.concatenate([[0], np.cumsum(w["block_partition"])])
    A = np.zeros((g.n, g.n))
    for e in range(g.nnz):
        r = w["edge_to_row"][e]; win = r // H
        c = w["edge_to_col"][e]
        cell = ((blk_base[win] + c // W) * H + (r % H)) * W + c % W
        tiles[cell] += 1
        A[r, w["win_cols"][w["win_col_ptr"][win] + c]] += 1
    assert tiles.sum() == g.nnz and tiles.max() == 1
    assert np.array_equal(A, dense_adj(g))


# ---------------------------------------------------------------- SpMM
@pytest.mark.parametrize("gi", range(5))
def test_spmm_dense_bruteforce(oracle, gi):
    g = small_graphs()[gi]
    rng = np.random.default_rng(100 + gi)
    vals = rng.standard_normal(g.nnz)
    X = rng.standard_normal((g.n, 7))
    out, ab = oracle.spmm(g.row_ptr, g.col_idx, vals, X)
    A = dense_adj(g, vals)
    assert np.allclose(out, A @ X, rtol=1e-12, atol=1e-13)
    assert np.allclose(ab, np.abs(A) @ np.abs(X), rtol=1e-12)   # no duplicate entries here
    # third opinion
    S = sp.csr_matrix((vals, g.col_idx, g.row_ptr), shape=(g.n, g.n))
    assert np.allclose(out, S @ X, rtol=1e-12, atol=1e-13)


def test_spmm_identity_and_unit_values(oracle):
    g = small_graphs()[2]
    out, _ = oracle.spmm(g.row_ptr, g.col_idx, None, np.eye(g.n))
    assert np.array_equal(out, dense_adj(g))


def test_spmm_duplicates_add_and_empty_rows_zero(oracle):
    rp = np.array([0, 3, 3, 4]); ci = np.array([2, 0, 2, 1])
    vals = np.array([1.0, 2.0, 4.0, -1.0])
    X = np.array([[1.0, 10.0], [2.0, 20.0], [3.0, 30.0]])
    out, ab = oracle.spmm(rp, ci, vals, X)
    assert np.array_equal(out, [[17.0, 170.0], [0, 0], [-2.0, -20.0]])
    assert np.array_equal(ab, [[17.0, 170.0], [0, 0], [2.0, 20.0]])


def test_spmm_not_transposed(oracle):
    # a directed pattern: only entry (0,1). out[0] = X[1], out[1] = 0.
    rp = np.array([0, 1, 1]); ci = np.array([1])
    out, _ = oracle.spmm(rp, ci, np.array([2.0]), np.array([[5.0], [7.0]]))
    assert np.array_equal(out, [[14.0], [0.0]])


# ---------------------------------------------------------------- SDDMM
@pytest.mark.parametrize("gi", range(5))
def test_sddmm_dense_bruteforce(oracle, gi):
    g = small_graphs()[gi]
    rng = np.random.default_rng(200 + gi)
    X = rng.standard_normal((g.n, 5)); Y = rng.standard_normal((g.n, 5))
    rs = rng.uniform(0.5, 2, g.n); cs = rng.uniform(0.5, 2, g.n)
    s, ab = oracle.sddmm(g.row_ptr, g.col_idx, X, Y, rs, cs, alpha=-1.5)
    full = -1.5 * (rs[:, None] * (X @ Y.T) * cs[None, :])
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    assert np.allclose(s, full[rows, g.col_idx], rtol=1e-12, atol=1e-13)
    fabs = 1.5 * (rs[:, None] * (np.abs(X) @ np.abs(Y).T) * cs[None, :])
    assert np.allclose(ab, fabs[rows, g.col_idx], rtol=1e-12)
    s1, _ = oracle.sddmm(g.row_ptr, g.col_idx, X, Y)
    assert np.allclose(s1, (X @ Y.T)[rows, g.col_idx], rtol=1e-12, atol=1e-13)


def test_sddmm_not_transposed(oracle):
    rp = np.array([0, 1, 1]); ci = np.array([1])
    X = np.array([[1.0, 2.0], [0.0, 0.0]]); Y = np.array([[9.0, 9.0], [3.0, 4.0]])
    s, _ = oracle.sddmm(rp, ci, X, Y, rs=np.array([2.0, 100.0]), cs=np.array([100.0, 5.0]))
    assert s[0] == 2.0 * 5.0 * 11.0


def test_agnn_scores_cosine_properties(oracle):
    g = small_graphs()[0]
    rng = np.random.default_rng(3)
    H = rng.standard_normal((g.n, 6))
    rinv = oracle.row_rnorm(H)
    assert np.allclose(np.linalg.norm(H * rinv[:, None], axis=1), 1.0, rtol=1e-14)
    beta = 1.7
    s, _ = oracle.sddmm(g.row_ptr, g.col_idx, H, H, rinv, rinv, beta)
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    assert np.all(np.abs(s) <= beta * (1 + 1e-14))
    assert np.allclose(s[rows == g.col_idx], beta, rtol=1e-14)      # self-loops: cos = 1
    S = np.zeros((g.n, g.n)); S[rows, g.col_idx] = s
    assert np.allclose(S, S.T, rtol=1e-14)                          # symmetric graph


def test_row_rnorm_zero_row(oracle):
    H = np.array([[0.0, 0.0], [3.0, 4.0]])
    rinv = oracle.row_rnorm(H)
    assert rinv[0] == 1e12 and rinv[1] == 0.2
    s, _ = oracle.sddmm(np.array([0, 2, 4]), np.array([0, 1, 0, 1]), H, H, rinv, rinv, 1.0)
    assert s[0] == 0 and s[1] == 0 and s[2] == 0 and abs(s[3] - 1) < 1e-15


# ---------------------------------------------------------------- edge softmax
@pytest.mark.parametrize("gi", range(5))
def test_softmax_invariants(oracle, gi):
    g = small_graphs()[gi]
    rng = np.random.default_rng(300 + gi)
    s = rng.standard_normal(g.nnz) * 3
    p = oracle.edge_softmax(g.row_ptr, s)
    deg = np.diff(g.row_ptr)
    rows = np.repeat(np.arange(g.n), deg)
    sums = np.bincount(rows, weights=p, minlength=g.n)
    assert np.allclose(sums[deg > 0], 1.0, atol=1e-12)
    assert np.all(p > 0)
    p2 = oracle.edge_softmax(g.row_ptr, s + 123.0)
    assert np.allclose(p, p2, rtol=1e-10)
    # direct definition with numpy, row by row
    for i in range(g.n):
        seg = s[g.row_ptr[i]:g.row_ptr[i + 1]]
        if seg.size:
            want = np.exp(seg) / np.exp(seg).sum()
            assert np.allclose(p[g.row_ptr[i]:g.row_ptr[i + 1]], want, rtol=1e-12)
    pe = oracle.edge_softmax(g.row_ptr, np.full(g.nnz, 0.37))
    assert np.allclose(pe, 1.0 / deg[rows], rtol=1e-14)


def test_softmax_large_scores_do_not_overflow(oracle):
    p = oracle.edge_softmax(np.array([0, 3]), np.array([1000.0, 1001.0, 999.0]))
    want = np.exp([-1.0, 0.0, -2.0]); want /= want.sum()
    assert np.allclose(p, want, rtol=1e-14)
    # a spread that only the shift by the row MAXIMUM survives (exp(1600) is no double)
    p = oracle.edge_softmax(np.array([0, 3]), np.array([800.0, -800.0, 799.0]))
    e = np.exp(-1.0)
    assert np.allclose(p, [1.0 / (1.0 + e), 0.0, e / (1.0 + e)], rtol=1e-14, atol=0)


# ---------------------------------------------------------------- layers
@pytest.mark.parametrize("gi", [0, 2, 3])
def test_gcn_layer_associativity_and_identity(oracle, gi):
    g = small_graphs()[gi]
    rng = np.random.default_rng(400 + gi)
    vals, _ = oracle.gcn_norm(g.row_ptr, g.col_idx)
    X = rng.standard_normal((g.n, 9)); W = rng.standard_normal((9, 4))
    out, ab = oracle.gcn_layer(g.row_ptr, g.col_idx, vals, X, W, relu=False)
    AX, _ = oracle.spmm(g.row_ptr, g.col_idx, vals, X)
    assert np.allclose(out, AX @ W, rtol=1e-11, atol=1e-12)
    A = dense_adj(g, vals)
    assert np.allclose(out, A @ (X @ W), rtol=1e-11, atol=1e-12)
    assert np.allclose(ab, np.abs(A) @ (np.abs(X) @ np.abs(W)), rtol=1e-11)
    outr, _ = oracle.gcn_layer(g.row_ptr, g.col_idx, vals, X, W, relu=True)
    assert np.array_equal(outr, np.maximum(out, 0))
    oi, _ = oracle.gcn_layer(g.row_ptr, g.col_idx, vals, X, np.eye(9))
    assert np.allclose(oi, AX, rtol=1e-14, atol=1e-15)


def test_gemm_not_transposed(oracle):
    X = np.array([[1.0, 2.0, 3.0]]); W = np.array([[1.0, 0.0], [0.0, 1.0], [10.0, 100.0]])
    Z, ab = oracle.gemm(X, W)
    assert np.array_equal(Z, [[31.0, 302.0]])
    rng = np.random.default_rng(0)
    X = rng.standard_normal((13, 6)); W = rng.standard_normal((6, 5))
    Z, ab = oracle.gemm(X, W)
    assert np.allclose(Z, X @ W, rtol=1e-13) and np.allclose(ab, np.abs(X) @ np.abs(W), rtol=1e-13)


def test_agnn_layer_hand_example(oracle):
    L = golden_lines("h2_agnn_path4.txt")
    H = np.array([[1, 0], [1, 1], [0, 2], [-1, 1.0]])
    for k in range(0, len(L), 6):
        beta = float(L[k])
        P = np.array([float(t) for t in L[k + 1].split()])
        PH = np.array([[float(t) for t in ln.split()] for ln in L[k + 2:k + 6]])
        out, _, p = oracle.agnn_layer(PATH_RP, PATH_CI, H, beta)
        assert np.allclose(p, P, atol=2e-6)
        assert np.allclose(out, PH, atol=2e-6)


@pytest.mark.parametrize("gi", [0, 2, 3, 4])
def test_agnn_layer_properties(oracle, gi):
    g = small_graphs()[gi]
    rng = np.random.default_rng(500 + gi)
    H = rng.standard_normal((g.n, 8))
    out, ab, p = oracle.agnn_layer(g.row_ptr, g.col_idx, H, beta=1.3)
    # dense re-derivation with numpy
    Hn = H / np.linalg.norm(H, axis=1, keepdims=True)
    S = 1.3 * Hn @ Hn.T
    M = dense_adj(g) > 0
    E = np.where(M, np.exp(S), 0.0)
    P = E / E.sum(1, keepdims=True)
    assert np.allclose(out, P @ H, rtol=1e-11, atol=1e-12)
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    assert np.allclose(p, P[rows, g.col_idx], rtol=1e-11)
    # convex combination of neighbour rows
    for i in range(g.n):
        nb = g.col_idx[g.row_ptr[i]:g.row_ptr[i + 1]]
        assert np.all(out[i] <= H[nb].max(0) + 1e-12) and np.all(out[i] >= H[nb].min(0) - 1e-12)
    # beta = 0: plain mean over stored neighbours (D^-1 A)
    out0, _, p0 = oracle.agnn_layer(g.row_ptr, g.col_idx, H, beta=0.0)
    deg = np.diff(g.row_ptr)
    assert np.allclose(p0, 1.0 / deg[rows], rtol=1e-14)
    assert np.allclose(out0, (dense_adj(g) / deg[:, None]) @ H, rtol=1e-12, atol=1e-13)
