"""Seeded synthetic graphs in CSR form.

The paper evaluates on citeseer, cora, amazon0505, com-amazon and amazon0601 (dataset
table, Section VI); those files are not available, so graphs of comparable shape are
generated instead: Erdos-Renyi, Chung-Lu power law, a permuted stochastic block model,
R-MAT, and a family whose row windows have a controlled tile fill.

Every generator returns an undirected graph stored as a directed CSR adjacency:
pairs with u == v dropped, both directions present, duplicates removed, optional
self-loops added, column indices ascending within each row.
"""
from dataclasses import dataclass

import numpy as np


@dataclass
class Graph:
    n: int
    row_ptr: np.ndarray  # int32 [n+1]
    col_idx: np.ndarray  # int32 [nnz]
    name: str = ""

    @property
    def nnz(self) -> int:
        return int(self.col_idx.shape[0])


def csr_from_pairs(n, u, v, self_loops=True, name=""):
    """Undirected pair list -> symmetric, deduplicated CSR with sorted columns."""
    u = np.asarray(u, dtype=np.int64)
    v = np.asarray(v, dtype=np.int64)
    keep = u != v
    u, v = u[keep], v[keep]
    parts = [u * n + v, v * n + u]
    if self_loops:
        d = np.arange(n, dtype=np.int64)
        parts.append(d * n + d)
    key = np.concatenate(parts)
    del parts
    key = np.unique(key)  # ascending => row-major order, columns ascending
    rows = key // n
    cols = (key - rows * n).astype(np.int32)
    counts = np.bincount(rows, minlength=n)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    assert row_ptr[-1] < 2**31
    return Graph(n, row_ptr.astype(np.int32), cols, name)


def erdos_renyi(n, m, seed, self_loops=True):
    """G(n, M): m uniformly random pairs."""
    rng = np.random.default_rng(seed)
    u = rng.integers(0, n, size=m)
    v = rng.integers(0, n, size=m)
    return csr_from_pairs(n, u, v, self_loops, f"er_n{n}")


def _chung_lu_weights(n, gamma, avg_deg):
    """w_i ~ (i + i0)^(-1/(gamma-1)), mean avg_deg, max sqrt(avg_deg * n)."""
    alpha = 1.0 / (gamma - 1.0)
    target = np.sqrt(avg_deg * n)
    idx = np.arange(n, dtype=np.float64)

    def wmax(i0):
        raw = (idx + i0) ** (-alpha)
        return avg_deg * n / raw.sum() * raw[0]

    lo, hi = 1e-6, float(n)
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if wmax(mid) > target:
            lo = mid
        else:
            hi = mid
    i0 = 0.5 * (lo + hi)
    raw = (idx + i0) ** (-alpha)
    return raw * (avg_deg * n / raw.sum())


def chung_lu(n, gamma, avg_deg, seed, self_loops=True, permute=True):
    """Chung-Lu power-law graph; every node ends with at least one neighbour."""
    rng = np.random.default_rng(seed)
    w = _chung_lu_weights(n, gamma, avg_deg)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    m = int(n * avg_deg / 2)
    u = np.searchsorted(cdf, rng.random(m), side="right")
    v = np.searchsorted(cdf, rng.random(m), side="right")
    np.minimum(u, n - 1, out=u)
    np.minimum(v, n - 1, out=v)
    deg = np.bincount(u[u != v], minlength=n) + np.bincount(v[u != v], minlength=n)
    lonely = np.nonzero(deg == 0)[0]
    if lonely.size:
        partner = np.minimum(np.searchsorted(cdf, rng.random(lonely.size), side="right"), n - 1)
        clash = partner == lonely
        partner[clash] = (partner[clash] + 1) % n
        u = np.concatenate([u, lonely])
        v = np.concatenate([v, partner])
    if permute:
        perm = rng.permutation(n)
        u, v = perm[u], perm[v]
    return csr_from_pairs(n, u, v, self_loops, f"chunglu_n{n}_g{gamma}")


def sbm(n_comm, comm_size, in_pairs, out_pairs, seed, self_loops=True, permute=True):
    """Stochastic block model sampled by pair count, node ids randomly permuted."""
    rng = np.random.default_rng(seed)
    n = n_comm * comm_size
    c = rng.integers(0, n_comm, size=in_pairs)
    u_in = c * comm_size + rng.integers(0, comm_size, size=in_pairs)
    v_in = c * comm_size + rng.integers(0, comm_size, size=in_pairs)
    us, vs = [u_in], [v_in]
    need = out_pairs
    while need > 0:
        a = rng.integers(0, n, size=int(need * 1.05) + 16)
        b = rng.integers(0, n, size=a.size)
        ok = (a // comm_size) != (b // comm_size)
        a, b = a[ok][:need], b[ok][:need]
        us.append(a)
        vs.append(b)
        need -= a.size
    u = np.concatenate(us)
    v = np.concatenate(vs)
    if permute:
        perm = rng.permutation(n)
        u, v = perm[u], perm[v]
    return csr_from_pairs(n, u, v, self_loops, f"sbm_n{n}")


def rmat(scale, samples_per_node, seed, a=0.57, b=0.19, c=0.19, self_loops=True):
    """R-MAT without noise; ids are not permuted (low ids are the hubs)."""
    rng = np.random.default_rng(seed)
    n = 1 << scale
    m = samples_per_node * n
    u = np.zeros(m, dtype=np.int64)
    v = np.zeros(m, dtype=np.int64)
    for _ in range(scale):
        r = rng.random(m)
        down = r >= a + b              # quadrants c, d: row bit set
        right = ((r >= a) & (r < a + b)) | (r >= a + b + c)  # quadrants b, d: column bit set
        u = (u << 1) | down
        v = (v << 1) | right
    return csr_from_pairs(n, u, v, self_loops, f"rmat_s{scale}")


def fill_controlled(n, pool, k, seed, blk_h=16, self_loops=False):
    """Each blk_h-row window draws `pool` distinct columns; every row takes k of them.

    The condensed tiles of a window then have fill close to k / pool.  The result is a
    directed pattern (not symmetrised): it is used for kernel sweeps, not for GCN.
    """
    rng = np.random.default_rng(seed)
    n_win = (n + blk_h - 1) // blk_h
    rows_out, cols_out = [], []
    k = min(k, pool)
    for w in range(n_win):
        cols = rng.choice(n, size=pool, replace=False)
        r0, r1 = w * blk_h, min(n, (w + 1) * blk_h)
        # every row of the window: k distinct members of the pool (k smallest of a random key)
        pick = np.argpartition(rng.random((r1 - r0, pool)), k - 1, axis=1)[:, :k] if k < pool else \
            np.tile(np.arange(pool), (r1 - r0, 1))
        rows_out.append(np.repeat(np.arange(r0, r1, dtype=np.int64), k))
        cols_out.append(cols[pick].reshape(-1))
    rows = np.concatenate(rows_out)
    cols = np.concatenate(cols_out)
    if self_loops:
        d = np.arange(n, dtype=np.int64)
        rows = np.concatenate([rows, d])
        cols = np.concatenate([cols, d])
    key = np.unique(rows * n + cols)
    rows = key // n
    cols = (key - rows * n).astype(np.int32)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=n), out=row_ptr[1:])
    return Graph(n, row_ptr.astype(np.int32), cols, f"fill_n{n}_u{pool}_k{k}")


# The five benchmark configurations.  `scale` < 1 shrinks the node count (same recipe)
# so the slow CPU oracle can check every element.
CONFIGS = {
    1: dict(kind="er", n=2048, seed=0),
    2: dict(kind="chung_lu", n=100_000, gamma=2.1, avg_deg=16, seed=1),
    3: dict(kind="chung_lu", n=200_000, gamma=2.3, avg_deg=20, seed=2),
    4: dict(kind="sbm", n_comm=1000, comm_size=1000, seed=3),
    5: dict(kind="rmat", scale=20, seed=4),
}


def config_graph(cfg, scale=1.0):
    """Graph of benchmark configuration `cfg` (1..5); scale shrinks the node count."""
    p = CONFIGS[cfg]
    if p["kind"] == "er":
        n = max(16, int(p["n"] * scale))
        return erdos_renyi(n, 4 * n, p["seed"])
    if p["kind"] == "chung_lu":
        n = max(64, int(p["n"] * scale))
        return chung_lu(n, p["gamma"], p["avg_deg"], p["seed"])
    if p["kind"] == "sbm":
        n_comm = max(2, int(round(p["n_comm"] * scale)))
        size = p["comm_size"]
        return sbm(n_comm, size, 14 * n_comm * size, 2 * n_comm * size, p["seed"])
    if p["kind"] == "rmat":
        s = p["scale"] + int(round(np.log2(scale))) if scale != 1.0 else p["scale"]
        return rmat(max(4, s), 16, p["seed"])
    raise ValueError(cfg)
