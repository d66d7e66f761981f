"""Pins of the reordering oracle: what the definition and the mathematics fix, not the oracle's own
code -- P A P^T against a dense permutation product, the permutation-in / permutation-out contract
against the forward oracle on the original graph, monotone keys, stability, hand-written cases."""
import numpy as np
import pytest

import synth
from oracle import ftc_oracle_reorder as R


def dense(n, row_ptr, col_idx):
    A = np.zeros((n, n))
    for i in range(n):
        for e in range(row_ptr[i], row_ptr[i + 1]):
            A[i, col_idx[e]] += 1.0           # duplicates count
    return A


def small_graph(seed, n=37, directed=True):
    rng = np.random.default_rng(seed)
    deg = rng.integers(0, 9, size=n)
    deg[3] = 0
    deg[11] = 30                              # a hub with duplicates
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    row_ptr[1:] = np.cumsum(deg)
    col = rng.integers(0, n, size=int(row_ptr[-1]))
    return n, row_ptr, col


def test_hand_written_case():
    # degrees 1, 3, 0, 3, 2  ->  order 1, 3 (tie by id), 4, 0, 2
    row_ptr = np.array([0, 1, 4, 4, 7, 9])
    col_idx = np.array([4, 0, 3, 1, 4, 1, 3, 0, 3])
    perm, inv = R.degree_order(row_ptr)
    assert perm.tolist() == [1, 3, 4, 0, 2]
    assert inv.tolist() == [3, 0, 4, 1, 2]
    rp, ci = R.permute_graph(row_ptr, col_idx, perm, inv)
    assert rp.tolist() == [0, 3, 6, 8, 9, 9]
    # row 0 = old row 1 = {0, 3, 1} -> {3, 1, 0} sorted {0, 1, 3}; row 1 = old 3 = {4, 1, 3} -> {2, 0, 1};
    # row 2 = old 4 = {0, 3} -> {3, 1}; row 3 = old 0 = {4} -> {2}
    assert ci.tolist() == [0, 1, 3, 0, 1, 2, 1, 3, 2]


def test_degree_classes_keep_the_original_order_inside_a_class():
    # degrees 5, 1, 4, 0, 7, 2, 3, 1: bit lengths 3, 1, 3, 0, 3, 2, 2, 1
    deg = np.array([5, 1, 4, 0, 7, 2, 3, 1])
    row_ptr = np.concatenate([[0], np.cumsum(deg)])
    perm, _ = R.degree_order(row_ptr, R.ORDER_DEGREE_CLASSES)
    assert perm.tolist() == [0, 2, 4, 5, 6, 1, 7, 3]
    assert R.bit_length(np.array([0, 1, 2, 3, 4, 7, 8, 1023, 1024])).tolist() == [0, 1, 2, 2, 3, 3, 4, 10, 11]


@pytest.mark.parametrize("mode", [R.ORDER_DEGREE, R.ORDER_DEGREE_CLASSES])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_relabelled_graph_is_the_permuted_matrix(mode, seed):
    n, row_ptr, col = small_graph(seed)
    perm, inv = R.degree_order(row_ptr, mode)
    assert sorted(perm.tolist()) == list(range(n)) and np.array_equal(inv[perm], np.arange(n))
    rp, ci = R.permute_graph(row_ptr, col, perm, inv)
    A = dense(n, row_ptr, col)
    Pm = np.zeros((n, n))
    Pm[np.arange(n), perm] = 1.0                      # (P A P^T)[a, b] = A[perm[a], perm[b]]
    assert np.array_equal(dense(n, rp, ci), Pm @ A @ Pm.T)
    for r in range(n):
        assert np.all(np.diff(ci[rp[r]:rp[r + 1]]) >= 0)          # ascending inside every row
    deg_new = np.diff(rp)
    key = deg_new if mode == R.ORDER_DEGREE else R.bit_length(deg_new)
    assert np.all(np.diff(key) <= 0)                               # keys never increase
    same = np.flatnonzero(np.diff(key) == 0)
    assert np.all(perm[same] < perm[same + 1])                     # ties: ascending old id


def test_permutation_in_permutation_out_contract(oracle):
    """Aggregating on the relabelled graph with relabelled features and mapping the result back
    equals aggregating on the original graph (each row's sum only changes its order of terms)."""
    g = synth.config_graph(2, 0.02)
    perm, inv = R.degree_order(g.row_ptr)
    rp, ci = R.permute_graph(g.row_ptr, g.col_idx, perm, inv)
    X = synth.normal_features(g.n, 8, seed=5).astype(np.float64)
    ref, _ = oracle.spmm(g.row_ptr, g.col_idx, None, X)
    Xp = R.permute_rows(X, perm)
    out_p, _ = oracle.spmm(rp.astype(np.int32), ci.astype(np.int32), None, Xp)
    back = R.permute_rows(out_p, inv)
    assert np.allclose(back, ref, rtol=1e-12, atol=1e-12)
    assert np.array_equal(R.permute_rows(R.permute_rows(X, perm), inv), X)


def test_degree_order_concentrates_the_columns_of_a_skewed_graph(oracle):
    """The purpose of the step: on a power-law graph whose ids carry no locality the windows of the
    relabelled graph hold fewer distinct columns in total."""
    g = synth.config_graph(2, 0.05)
    perm, inv = R.degree_order(g.row_ptr)
    rp, ci = R.permute_graph(g.row_ptr, g.col_idx, perm, inv)
    before = oracle.build_windows(g.row_ptr, g.col_idx)["summary"][0]
    after = oracle.build_windows(rp.astype(np.int32), ci.astype(np.int32))["summary"][0]
    assert after < before


def csr_of(n, pairs):
    rows = [[] for _ in range(n)]
    for a, b in pairs:
        rows[a].append(b)
    row_ptr = np.concatenate([[0], np.cumsum([len(r) for r in rows])])
    col = np.array([c for r in rows for c in r], dtype=np.int64)
    return row_ptr, col


def test_label_propagation_hand_worked_round():
    # path 0 - 1 - 2 with self-loops, plus node 3 without entries and node 4 pointing twice at 2 and once at 0
    row_ptr, col = csr_of(5, [(0, 0), (0, 1), (1, 0), (1, 1), (1, 2), (2, 1), (2, 2), (4, 2), (4, 2), (4, 0)])
    # round 1 from labels 0..4: node 0 sees {0, 1} -> tie -> 0; node 1 sees {0, 1, 2} -> 0; node 2 sees {1, 2} -> 1;
    # node 3 keeps 3; node 4 sees {2, 2, 0} -> 2
    assert R.label_propagation(row_ptr, col, 1).tolist() == [0, 0, 1, 3, 2]
    # round 2 from [0, 0, 1, 3, 2]: node 0 sees {0, 0} -> 0; node 1 sees {0, 0, 1} -> 0; node 2 sees {0, 1} -> 0;
    # node 4 sees {1, 1, 0} -> 1
    assert R.label_propagation(row_ptr, col, 2).tolist() == [0, 0, 0, 3, 1]
    assert R.label_propagation(row_ptr, col, 0).tolist() == [0, 1, 2, 3, 4]


def test_label_propagation_separates_disjoint_cliques():
    a, b = [0, 2, 4, 6, 8], [1, 3, 5, 7, 9, 10]
    pairs = [(u, v) for grp in (a, b) for u in grp for v in grp]
    row_ptr, col = csr_of(11, pairs)
    lab = R.label_propagation(row_ptr, col, 3)
    assert set(lab[a]) == {0} and set(lab[b]) == {1}


def test_label_propagation_recovers_a_planted_partition():
    """Stochastic block model with permuted ids: after ten rounds nearly every node carries the label of
    its planted community (the generator's permutation is undone through the edges themselves: two
    nodes joined by an in-community edge get the same label)."""
    g = synth.sbm(12, 200, 14 * 12 * 200, 2 * 12 * 200, seed=5)
    lab = R.label_propagation(g.row_ptr, g.col_idx, 10)
    values, counts = np.unique(lab, return_counts=True)
    big = values[counts >= 100]
    assert big.size == 12                                   # one label per planted community ...
    assert counts[counts >= 100].sum() >= 0.97 * g.n        # ... holding nearly all nodes
    rows = np.repeat(np.arange(g.n), np.diff(g.row_ptr))
    same = lab[rows] == lab[g.col_idx]
    assert same.mean() > 0.85                               # 14 of 16 sampled pairs are in-community


def test_order_by_key_groups_equal_keys_and_keeps_their_order():
    keys = np.array([7, 3, 7, 0, 3, 3, 9, 0])
    perm, inv = R.order_by_key(keys)
    assert perm.tolist() == [3, 7, 1, 4, 5, 0, 2, 6]
    assert np.array_equal(inv[perm], np.arange(8))
