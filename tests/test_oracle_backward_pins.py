"""Pins of the backward oracle (CPU only): central finite differences of the FORWARD oracle (the C
routines, which have their own pins), closed-form special cases, and the transposed index against a
dense transpose."""
import numpy as np
import pytest

import synth
from oracle import ftc_oracle_backward as ob


def small_graph(seed, n=14, m=30, symmetric=True):
    g = synth.erdos_renyi(n, m, seed=seed)          # symmetrised, de-duplicated, with self-loops
    if symmetric:
        return g
    # drop some entries to break the symmetry of the pattern (the oracle must not rely on it)
    rng = np.random.default_rng(seed)
    keep = rng.random(g.nnz) > 0.3
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    keep |= rows == g.col_idx                        # keep the self-loops: no empty rows
    rp = np.zeros(g.n + 1, dtype=np.int32)
    rp[1:] = np.cumsum(np.bincount(rows[keep], minlength=g.n))
    return synth.Graph(g.n, rp, g.col_idx[keep].astype(np.int32))


def fd(f, x, eps=1e-6):
    """Central differences of the scalar function f at the array x."""
    grad = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        old = x[idx]
        x[idx] = old + eps
        up = f()
        x[idx] = old - eps
        dn = f()
        x[idx] = old
        grad[idx] = (up - dn) / (2 * eps)
    return grad


@pytest.mark.parametrize("seed", [0, 1])
@pytest.mark.parametrize("symmetric", [True, False])
@pytest.mark.parametrize("relu", [False, True])
def test_gcn_backward_matches_finite_differences(oracle, seed, symmetric, relu):
    g = small_graph(seed, symmetric=symmetric)
    rng = np.random.default_rng(10 + seed)
    vals = rng.uniform(0.2, 1.0, g.nnz)
    X = rng.standard_normal((g.n, 5))
    W = rng.standard_normal((5, 3))
    R = rng.standard_normal((g.n, 3))                # loss = sum(Y * R), so dL/dY = R

    def loss():
        Y, _ = oracle.gcn_layer(g.row_ptr, g.col_idx, vals, X, W, relu=relu)
        return float((Y * R).sum())

    Y, _ = oracle.gcn_layer(g.row_ptr, g.col_idx, vals, X, W, relu=relu)
    assert not relu or np.min(np.abs(Y[Y != 0])) > 1e-4   # no output sits on the kink of the ReLU
    dX, dW, _ = ob.gcn_layer_backward(g.row_ptr, g.col_idx, vals, X, W, R, Y if relu else None)
    assert np.allclose(dX, fd(loss, X), rtol=1e-6, atol=1e-7)
    assert np.allclose(dW, fd(loss, W), rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("symmetric", [True, False])
@pytest.mark.parametrize("beta", [1.0, -2.5, 0.0])
def test_agnn_backward_matches_finite_differences(oracle, seed, symmetric, beta):
    g = small_graph(seed, symmetric=symmetric)
    rng = np.random.default_rng(20 + seed)
    H = rng.standard_normal((g.n, 4))
    R = rng.standard_normal((g.n, 4))
    b = np.array([beta])

    def loss():
        Y, _, _ = oracle.agnn_layer(g.row_ptr, g.col_idx, H, float(b[0]))
        return float((Y * R).sum())

    dH, dbeta = ob.agnn_layer_backward(g.row_ptr, g.col_idx, H, beta, R)
    assert np.allclose(dH, fd(loss, H), rtol=2e-6, atol=1e-7)
    assert np.isclose(dbeta, fd(loss, b)[0], rtol=2e-6, atol=1e-7)


def test_agnn_backward_of_a_row_below_the_norm_clamp(oracle):
    """|h_i| <= 1e-12: the forward pass scales the row by 1e12 instead of normalising it, so the row enters
    linearly and its gradient has no projection term.  Central differences with a step far below the row's
    own size (the forward oracle is smooth there) pin exactly that."""
    g = small_graph(1, symmetric=True)
    rng = np.random.default_rng(31)
    H = rng.standard_normal((g.n, 4))
    R = rng.standard_normal((g.n, 4))
    i = 5
    H[i] = 5e-13 * rng.standard_normal(4) / 2.0
    assert np.linalg.norm(H[i]) < 1e-12 and g.row_ptr[i + 1] > g.row_ptr[i]

    def loss():
        Y, _, _ = oracle.agnn_layer(g.row_ptr, g.col_idx, H, 1.5)
        return float((Y * R).sum())

    dH, _ = ob.agnn_layer_backward(g.row_ptr, g.col_idx, H, 1.5, R)
    row = H[i:i + 1]                                   # a view: fd() perturbs H in place
    num = fd(loss, row, eps=1e-16)
    assert np.abs(num).max() > 1e9                     # the 1e12 scaling is visible
    assert np.allclose(dH[i], num[0], rtol=1e-5)
    others = np.delete(np.arange(g.n), i)
    assert np.allclose(dH[others], fd(loss, H)[others], rtol=2e-6, atol=1e-7)


def test_agnn_backward_beta_zero_is_mean_aggregation():
    """beta = 0: P = D^-1 A does not depend on H, so dH = P^T dY exactly (dense check)."""
    g = small_graph(3)
    rng = np.random.default_rng(5)
    H, R = rng.standard_normal((g.n, 3)), rng.standard_normal((g.n, 3))
    P = np.zeros((g.n, g.n))
    for i in range(g.n):
        cols = g.col_idx[g.row_ptr[i]:g.row_ptr[i + 1]]
        P[i, cols] = 1.0 / cols.size
    dH, _ = ob.agnn_layer_backward(g.row_ptr, g.col_idx, H, 0.0, R)
    assert np.allclose(dH, P.T @ R, atol=1e-13)


def test_gcn_backward_identity_weight_is_transposed_aggregation():
    g = small_graph(4, symmetric=False)
    rng = np.random.default_rng(6)
    vals = rng.uniform(0.2, 1.0, g.nnz)
    A = np.zeros((g.n, g.n))
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    A[rows, g.col_idx] = vals
    X, R = rng.standard_normal((g.n, 4)), rng.standard_normal((g.n, 4))
    dX, dW, dZ = ob.gcn_layer_backward(g.row_ptr, g.col_idx, vals, X, np.eye(4), R)
    assert np.allclose(dX, A.T @ R, atol=1e-13) and np.allclose(dZ, dX)
    assert np.allclose(dW, X.T @ (A.T @ R), atol=1e-12)


def test_softmax_backward_properties():
    g = small_graph(7)
    rng = np.random.default_rng(8)
    p = rng.random(g.nnz)
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    p /= np.bincount(rows, weights=p)[rows]
    dp = rng.standard_normal(g.nnz)
    ds = ob.edge_softmax_backward(g.row_ptr, p, dp)
    assert np.allclose(np.bincount(rows, weights=ds), 0, atol=1e-14)          # softmax is shift invariant
    assert np.allclose(ob.edge_softmax_backward(g.row_ptr, p, dp + 3.0), ds)   # ... so a row constant drops out
    # Jacobian of a single row written out: diag(p) - p p^T
    i = int(np.argmax(np.diff(g.row_ptr)))
    sl = slice(g.row_ptr[i], g.row_ptr[i + 1])
    J = np.diag(p[sl]) - np.outer(p[sl], p[sl])
    assert np.allclose(ds[sl], J @ dp[sl])


@pytest.mark.parametrize("seed", [0, 1])
def test_transpose_index_against_dense(seed):
    g = small_graph(seed, n=20, m=50)
    T = ob.transpose_index(g.row_ptr, g.col_idx)
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    assert np.all(T >= 0)
    assert np.array_equal(rows[T], g.col_idx) and np.array_equal(g.col_idx[T], rows)
    assert np.array_equal(T[T], np.arange(g.nnz))
    gu = small_graph(seed, n=20, m=50, symmetric=False)
    Tu = ob.transpose_index(gu.row_ptr, gu.col_idx)
    dense = np.zeros((gu.n, gu.n), dtype=bool)
    ru = np.repeat(np.arange(gu.n), np.diff(gu.row_ptr))
    dense[ru, gu.col_idx] = True
    assert np.array_equal(Tu >= 0, dense.T[ru, gu.col_idx])


@pytest.mark.parametrize("beta", [1.0, -3.0, 0.0])
def test_row_z_is_the_denominator_of_the_forward_oracles_probabilities(oracle, beta):
    """p_e * z_i = exp(beta * c_e - |beta|) with p from the C forward oracle (independent code) and
    c_e from its SDDMM on the normalised rows; a row of identical neighbours has z = deg * exp(beta - |beta|)."""
    g = synth.config_graph(1)
    H = synth.normal_features(g.n, 12, seed=3).astype(np.float64)
    _, _, p = oracle.agnn_layer(g.row_ptr, g.col_idx, H, beta)
    Hn = H / np.sqrt((H * H).sum(axis=1))[:, None]
    c, _ = oracle.sddmm(g.row_ptr, g.col_idx, Hn, Hn)
    z = ob.agnn_row_z(g.row_ptr, g.col_idx, H, beta)
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    assert np.allclose(p * z[rows], np.exp(beta * c - abs(beta)), rtol=1e-12, atol=0)
    same = np.tile(H[:1], (g.n, 1))                      # every cosine is 1
    z1 = ob.agnn_row_z(g.row_ptr, g.col_idx, same, beta)
    assert np.allclose(z1, np.diff(g.row_ptr) * np.exp(beta - abs(beta)), rtol=1e-12)


@pytest.mark.parametrize("relu", [False, True])
def test_update_gemm_backward_against_finite_differences(oracle, relu):
    """Central differences of the forward C oracle's dense product (with the ReLU applied here)."""
    rng = np.random.default_rng(11)
    n, d_in, d_out = 9, 5, 4
    X, W = rng.normal(size=(n, d_in)), rng.normal(size=(d_in, d_out))
    dZ = rng.normal(size=(n, d_out))

    def loss(Xv, Wv):
        Z, _ = oracle.gemm(Xv, Wv)
        return float(((np.maximum(Z, 0) if relu else Z) * dZ).sum())

    Z0, _ = oracle.gemm(X, W)
    dX, dW = ob.update_gemm_backward(X, W, dZ, np.maximum(Z0, 0) if relu else None)
    eps = 1e-6
    for (i, j) in [(0, 0), (3, 2), (8, 4)]:
        Xp, Xm = X.copy(), X.copy()
        Xp[i, j] += eps
        Xm[i, j] -= eps
        assert dX[i, j] == pytest.approx((loss(Xp, W) - loss(Xm, W)) / (2 * eps), rel=1e-6, abs=1e-8)
    for (a, b) in [(0, 0), (2, 3), (4, 1)]:
        Wp, Wm = W.copy(), W.copy()
        Wp[a, b] += eps
        Wm[a, b] -= eps
        assert dW[a, b] == pytest.approx((loss(X, Wp) - loss(X, Wm)) / (2 * eps), rel=1e-6, abs=1e-8)


# ---- the yardsticks (sums of absolute terms) of the gradients --------------------------------------
def test_agnn_backward_terms_single_node_closed_form():
    """One node with a self-loop, h = (3, 4), dY = (1, -2), beta = 2, worked by hand: |h| = 5,
    hn = (0.6, 0.8), p = 1, sum |dY h| = 11 (twice: once as dp, once as the row sum), so the terms of
    ds add up to 22 and those of dbeta to 22 * 1; the terms of dhn are 2 * 22 * hn from each of the two
    roles of the loop, (52.8, 70.4), their projection onto |hn| is 88, and
    dH_terms = |dY| + (dhn_terms + |hn| * 88) / 5 = (22.12, 30.16)."""
    rp, ci = np.array([0, 1]), np.array([0])
    H, dY = np.array([[3.0, 4.0]]), np.array([[1.0, -2.0]])
    terms, dbeta_terms = ob.agnn_layer_backward_terms(rp, ci, H, 2.0, dY)
    assert np.allclose(terms, [[22.12, 30.16]], rtol=1e-12)
    assert abs(dbeta_terms - 22.0) < 1e-12
    dH, dbeta = ob.agnn_layer_backward(rp, ci, H, 2.0, dY)
    assert np.allclose(dH, dY) and abs(dbeta) < 1e-15        # softmax of one entry: only the aggregated part is left


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_backward_terms_bound_the_gradients_and_scale_with_them(oracle, seed):
    """Triangle inequality: every yardstick is at least the size of the value it belongs to; it does not
    change when the incoming gradient changes sign and scales with its size; with non-negative data and
    no subtraction in the chain (GCN without ReLU) it equals the value."""
    g = small_graph(seed, symmetric=bool(seed & 1))
    rng = np.random.default_rng(30 + seed)
    H = rng.standard_normal((g.n, 4))
    dY = rng.standard_normal((g.n, 4))
    dH, dbeta = ob.agnn_layer_backward(g.row_ptr, g.col_idx, H, -1.7, dY)
    tH, tb = ob.agnn_layer_backward_terms(g.row_ptr, g.col_idx, H, -1.7, dY)
    assert np.all(tH >= np.abs(dH) * (1 - 1e-12)) and tb >= abs(dbeta)
    tH2, tb2 = ob.agnn_layer_backward_terms(g.row_ptr, g.col_idx, H, -1.7, -3.0 * dY)
    assert np.allclose(tH2, 3.0 * tH, rtol=1e-12) and np.isclose(tb2, 3.0 * tb, rtol=1e-12)
    # an incoming yardstick larger than |dY| gives larger yardsticks (it is carried through linearly)
    tH3, _ = ob.agnn_layer_backward_terms(g.row_ptr, g.col_idx, H, -1.7, dY, dY_terms=2.0 * np.abs(dY))
    assert np.allclose(tH3, 2.0 * tH, rtol=1e-12)

    vals = rng.uniform(-1.0, 1.0, g.nnz)
    X, W, R = rng.standard_normal((g.n, 5)), rng.standard_normal((5, 3)), rng.standard_normal((g.n, 3))
    Y, _ = oracle.gcn_layer(g.row_ptr, g.col_idx, vals, X, W, relu=True)
    dX, dW, dZ = ob.gcn_layer_backward(g.row_ptr, g.col_idx, vals, X, W, R, Y)
    tX, tW, tZ = ob.gcn_layer_backward_terms(g.row_ptr, g.col_idx, vals, X, W, R, Y)
    for v, t in ((dX, tX), (dW, tW), (dZ, tZ)):
        assert np.all(t >= np.abs(v) * (1 - 1e-12))
    pos = [np.abs(a) for a in (vals, X, W, R)]
    dXp, dWp, dZp = ob.gcn_layer_backward(g.row_ptr, g.col_idx, *pos)
    tXp, tWp, tZp = ob.gcn_layer_backward_terms(g.row_ptr, g.col_idx, *pos)
    assert np.allclose(dXp, tXp, rtol=1e-12) and np.allclose(dWp, tWp, rtol=1e-12) and np.allclose(dZp, tZp, rtol=1e-12)
    dXu, dWu = ob.update_gemm_backward(X, W, R, Y)
    tXu, tWu = ob.update_gemm_backward_terms(X, W, R, Y)
    assert np.all(tXu >= np.abs(dXu) * (1 - 1e-12)) and np.all(tWu >= np.abs(dWu) * (1 - 1e-12))
    assert np.allclose(ob.update_gemm_backward_terms(pos[1], pos[2], pos[3])[1], pos[1].T @ pos[3], rtol=1e-12)
