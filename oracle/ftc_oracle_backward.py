"""fp64 CPU oracle of the BACKWARD pass of the two layers (TEST INFRASTRUCTURE ONLY).

The paper speaks of GNN training and inference (Sections II and V) but gives no gradient
formulas; these are the derivatives of the forward definitions in ftc_oracle.c, written out with
numpy as plain sums over the stored entries.  No symmetry of the pattern is assumed: products with
a transposed sparse matrix are scatters (numpy.add.at) over the entries of the untransposed one.
Nothing in the product library imports this file, and it shares no code with the HIP kernels.

Notation: e = (i, j) is a stored entry of row i with column j = col_idx[e]; rows[e] = i.
"""
import numpy as np


def _rows(row_ptr):
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    return np.repeat(np.arange(row_ptr.size - 1), np.diff(row_ptr))


def transpose_index(row_ptr, col_idx):
    """T[e] = index of the entry (j, i) for e = (i, j), or -1 if the pattern does not hold it.
    Requires ascending, duplicate-free columns inside every row."""
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    col = np.asarray(col_idx, dtype=np.int64)
    rows = _rows(row_ptr)
    T = np.full(col.size, -1, dtype=np.int64)
    for e in range(col.size):
        i, j = rows[e], col[e]
        lo, hi = row_ptr[j], row_ptr[j + 1]
        k = lo + np.searchsorted(col[lo:hi], i)
        if k < hi and col[k] == i:
            T[e] = k
    return T


def gcn_layer_backward(row_ptr, col_idx, vals, X, W, dY, Y=None):
    """Forward: Z = X W, P = A^ Z, Y = relu(P) (or Y = P when Y is None here).
    Returns (dX [n, d_in], dW [d_in, d_out], dZ [n, d_out]) for a loss with dL/dY = dY:
      dP = dY where Y > 0 (ReLU) else 0;  dZ = A^T dP;  dW = X^T dZ;  dX = dZ W^T."""
    col = np.asarray(col_idx, dtype=np.int64)
    rows = _rows(row_ptr)
    vals = np.ones(col.size) if vals is None else np.asarray(vals, dtype=np.float64)
    X, W, dY = (np.asarray(a, dtype=np.float64) for a in (X, W, dY))
    dP = dY if Y is None else dY * (np.asarray(Y, dtype=np.float64) > 0)
    dZ = np.zeros_like(dP)
    np.add.at(dZ, col, vals[:, None] * dP[rows])          # (A^T dP)[j] = sum over e = (i, j) of a_e dP[i]
    return dZ @ W.T, X.T @ dZ, dZ


def update_gemm_backward(X, W, dZ, Z=None):
    """Dense update Z = act(X W) (act = ReLU when Z, the layer's output, is given; identity otherwise).
    Returns (dX [n, d_in], dW [d_in, d_out]) for a loss with dL/dZ = dZ:
      dP = dZ where Z > 0 (ReLU) else dZ;  dW = X^T dP;  dX = dP W^T."""
    X, W, dZ = (np.asarray(a, dtype=np.float64) for a in (X, W, dZ))
    dP = dZ if Z is None else dZ * (np.asarray(Z, dtype=np.float64) > 0)
    return dP @ W.T, X.T @ dP


def edge_softmax_backward(row_ptr, p, dp):
    """ds[e] = p[e] * (dp[e] - sum over the row of p * dp): derivative of the row-wise softmax."""
    rows = _rows(row_ptr)
    p, dp = np.asarray(p, dtype=np.float64), np.asarray(dp, dtype=np.float64)
    n = np.asarray(row_ptr).size - 1
    rowsum = np.zeros(n)
    np.add.at(rowsum, rows, p * dp)
    return p * (dp - rowsum[rows])


def agnn_row_z(row_ptr, col_idx, H, beta):
    """z_i = sum over row i of exp(beta * c_e - |beta|): the softmax denominators in the form the
    single-pass forward keeps them for the backward pass (|c| <= 1, so |beta| bounds every score).
    0 for a row without entries."""
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    col = np.asarray(col_idx, dtype=np.int64)
    rows = _rows(row_ptr)
    H = np.asarray(H, dtype=np.float64)
    Hn = H / np.maximum(np.sqrt((H * H).sum(axis=1)), 1e-12)[:, None]
    c = (Hn[rows] * Hn[col]).sum(axis=1)
    z = np.zeros(H.shape[0])
    np.add.at(z, rows, np.exp(beta * c - abs(beta)))
    return z


def agnn_layer_backward(row_ptr, col_idx, H, beta, dY):
    """Forward: hn_i = h_i / max(|h_i|, 1e-12), c_e = <hn_i, hn_j>, p = row softmax of beta * c,
    y_i = sum_e p_e h_j.  Returns (dH [n, D], dbeta) for a loss with dL/dY = dY."""
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    col = np.asarray(col_idx, dtype=np.int64)
    rows = _rows(row_ptr)
    H, dY = np.asarray(H, dtype=np.float64), np.asarray(dY, dtype=np.float64)
    n = H.shape[0]
    nrm = np.sqrt((H * H).sum(axis=1))
    clamped = nrm <= 1e-12
    rinv = 1.0 / np.maximum(nrm, 1e-12)
    Hn = H * rinv[:, None]
    c = (Hn[rows] * Hn[col]).sum(axis=1)
    s = beta * c
    m = np.full(n, -np.inf)
    np.maximum.at(m, rows, s)
    ex = np.exp(s - m[rows])
    z = np.zeros(n)
    np.add.at(z, rows, ex)
    p = ex / z[rows]
    # y_i = sum_e p_e h_j
    dp = (dY[rows] * H[col]).sum(axis=1)
    dH = np.zeros_like(H)
    np.add.at(dH, col, p[:, None] * dY[rows])             # through the aggregated rows h_j
    ds = edge_softmax_backward(row_ptr, p, dp)
    dbeta = float((ds * c).sum())
    dc = beta * ds
    dHn = np.zeros_like(H)
    np.add.at(dHn, rows, dc[:, None] * Hn[col])           # c_e depends on hn_i ...
    np.add.at(dHn, col, dc[:, None] * Hn[rows])           # ... and on hn_j
    # hn = h / |h|:  dh = (dhn - hn <hn, dhn>) / |h|;  a clamped row is h * 1e12: no projection
    proj = (Hn * dHn).sum(axis=1)
    proj[clamped] = 0.0
    dH += rinv[:, None] * (dHn - Hn * proj[:, None])
    return dH, dbeta


# ---- error denominators -------------------------------------------------------------------------------
# The forward oracle returns, next to every sum, the sum of the absolute values of its terms: the
# yardstick an fp32 evaluation is measured against (a result that is small only because its terms
# cancel is not held to its own size).  The functions below give the same yardstick for the gradients:
# the backward formulas above evaluated with every factor replaced by its absolute value and every
# subtraction by an addition, carried through the chain (a running bound of the terms).  `dY_terms`
# is the yardstick of the incoming gradient when that is itself a computed quantity (a layer stack);
# by default the incoming gradient is exact data and its yardstick is |dY|.

def gcn_layer_backward_terms(row_ptr, col_idx, vals, X, W, dY, Y=None, dY_terms=None):
    """Yardsticks (dX_terms, dW_terms, dZ_terms) of gcn_layer_backward's three results."""
    col = np.asarray(col_idx, dtype=np.int64)
    rows = _rows(row_ptr)
    vals = np.ones(col.size) if vals is None else np.abs(np.asarray(vals, dtype=np.float64))
    X, W = np.abs(np.asarray(X, dtype=np.float64)), np.abs(np.asarray(W, dtype=np.float64))
    dP = np.abs(np.asarray(dY, dtype=np.float64)) if dY_terms is None else np.asarray(dY_terms, dtype=np.float64)
    if Y is not None:
        dP = dP * (np.asarray(Y, dtype=np.float64) > 0)
    dZ = np.zeros_like(dP)
    np.add.at(dZ, col, vals[:, None] * dP[rows])
    return dZ @ W.T, X.T @ dZ, dZ


def update_gemm_backward_terms(X, W, dZ, Z=None, dZ_terms=None):
    """Yardsticks (dX_terms, dW_terms) of update_gemm_backward's two results."""
    X, W = np.abs(np.asarray(X, dtype=np.float64)), np.abs(np.asarray(W, dtype=np.float64))
    dP = np.abs(np.asarray(dZ, dtype=np.float64)) if dZ_terms is None else np.asarray(dZ_terms, dtype=np.float64)
    if Z is not None:
        dP = dP * (np.asarray(Z, dtype=np.float64) > 0)
    return dP @ W.T, X.T @ dP


def agnn_layer_backward_terms(row_ptr, col_idx, H, beta, dY, dY_terms=None):
    """Yardsticks (dH_terms [n, D], dbeta_terms) of agnn_layer_backward's two results."""
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    col = np.asarray(col_idx, dtype=np.int64)
    rows = _rows(row_ptr)
    H = np.asarray(H, dtype=np.float64)
    aY = np.abs(np.asarray(dY, dtype=np.float64)) if dY_terms is None else np.asarray(dY_terms, dtype=np.float64)
    n = H.shape[0]
    nrm = np.sqrt((H * H).sum(axis=1))
    clamped = nrm <= 1e-12
    rinv = 1.0 / np.maximum(nrm, 1e-12)
    Hn = H * rinv[:, None]
    aH, aHn = np.abs(H), np.abs(Hn)
    c = (Hn[rows] * Hn[col]).sum(axis=1)
    c_terms = (aHn[rows] * aHn[col]).sum(axis=1)
    s = beta * c
    m = np.full(n, -np.inf)
    np.maximum.at(m, rows, s)
    ex = np.exp(s - m[rows])
    z = np.zeros(n)
    np.add.at(z, rows, ex)
    p = ex / z[rows]                                        # positive: its own yardstick
    dp_terms = (aY[rows] * aH[col]).sum(axis=1)
    t_terms = np.zeros(n)
    np.add.at(t_terms, rows, p * dp_terms)
    ds_terms = p * (dp_terms + t_terms[rows])
    dbeta_terms = float((ds_terms * c_terms).sum())
    dHn_terms = np.zeros_like(H)
    np.add.at(dHn_terms, rows, abs(beta) * ds_terms[:, None] * aHn[col])
    np.add.at(dHn_terms, col, abs(beta) * ds_terms[:, None] * aHn[rows])
    proj_terms = (aHn * dHn_terms).sum(axis=1)
    proj_terms[clamped] = 0.0
    dH_terms = np.zeros_like(H)
    np.add.at(dH_terms, col, p[:, None] * aY[rows])
    dH_terms += rinv[:, None] * (dHn_terms + aHn * proj_terms[:, None])
    return dH_terms, dbeta_terms
