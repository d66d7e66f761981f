"""CPU oracle of the locality reordering used in preprocessing (TEST INFRASTRUCTURE ONLY).

The paper's sparse graph transformation condenses the columns of a row window (Section IV.A); how
many columns the rows of a window share depends on the numbering of the nodes, which the paper
takes as given.  Relabelling the nodes before the transformation is the preprocessing step defined
here: a permutation of the node ids, the relabelled CSR, and the row maps that carry features into
the new numbering and results back (permutation in, permutation out).  Everything is integer work
with a unique result, written as plain loops and numpy sorts.  Nothing in the product library
imports this file, and it shares no code with the HIP kernels.

perm[new] = old id of the node that gets the id `new`;  inv[old] = new.
"""
import numpy as np

ORDER_DEGREE = 0          # descending number of stored entries of the row, ties by ascending id
ORDER_DEGREE_CLASSES = 1  # descending bit length of that number, ties by ascending id


def bit_length(x):
    """Number of bits of x (0 for 0): the power-of-two class of a degree."""
    x = np.asarray(x, dtype=np.int64)
    out = np.zeros(x.shape, dtype=np.int64)
    v = x.copy()
    while np.any(v > 0):
        out += v > 0
        v >>= 1
    return out


def degree_order(row_ptr, mode=ORDER_DEGREE):
    """(perm, inv) of the ordering `mode`."""
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    deg = np.diff(row_ptr)
    key = deg if mode == ORDER_DEGREE else bit_length(deg)
    n = deg.size
    perm = np.array(sorted(range(n), key=lambda i: (-int(key[i]), i)), dtype=np.int64)
    inv = np.empty(n, dtype=np.int64)
    inv[perm] = np.arange(n)
    return perm, inv


def permute_graph(row_ptr, col_idx, perm, inv):
    """CSR of the relabelled graph: row `new` holds the entries of row perm[new] with every column c
    replaced by inv[c], in ascending order (duplicates kept)."""
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    col = np.asarray(col_idx, dtype=np.int64)
    n = row_ptr.size - 1
    rp = np.zeros(n + 1, dtype=np.int64)
    out = []
    for new in range(n):
        old = perm[new]
        cols = np.sort(inv[col[row_ptr[old]:row_ptr[old + 1]]])
        out.append(cols)
        rp[new + 1] = rp[new] + cols.size
    ci = np.concatenate(out) if out else np.zeros(0, dtype=np.int64)
    return rp, ci.astype(np.int64)


def permute_rows(X, index):
    """out[r] = X[index[r]]: index = perm carries rows into the new numbering, index = inv back."""
    return np.asarray(X)[np.asarray(index, dtype=np.int64)]


def order_by_key(keys):
    """(perm, inv) of the ascending order of `keys`, ties by ascending id: nodes with the same key (for
    instance the same community label) become neighbours in the new numbering."""
    keys = np.asarray(keys, dtype=np.int64)
    n = keys.size
    perm = np.array(sorted(range(n), key=lambda i: (int(keys[i]), i)), dtype=np.int64)
    inv = np.empty(n, dtype=np.int64)
    inv[perm] = np.arange(n)
    return perm, inv


def label_propagation(row_ptr, col_idx, iters):
    """Synchronous label propagation, the community heuristic behind the community ordering: every node
    starts with its own id as label; in each of `iters` rounds every node takes the label that occurs
    most often among the stored entries of its row (duplicates count, a self-loop counts the node's
    own label), the smallest such label on a tie, all nodes at once from the labels of the previous
    round.  A node without entries keeps its label.  Returns the labels after the last round."""
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    col = np.asarray(col_idx, dtype=np.int64)
    n = row_ptr.size - 1
    label = np.arange(n, dtype=np.int64)
    for _ in range(iters):
        new = label.copy()
        for i in range(n):
            nb = label[col[row_ptr[i]:row_ptr[i + 1]]]
            if nb.size == 0:
                continue
            values, counts = np.unique(nb, return_counts=True)     # values ascending
            new[i] = values[np.argmax(counts)]                      # first maximum = smallest label
        label = new
    return label
