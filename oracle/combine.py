"""Oracle: weighted un-permute / combine (test infrastructure, CPU only).

Stands where the return all-to-all after the FFN layers is (Background, "The same
amount of communication happens for All-to-All shuffle after the FFN layers"):
each token gathers the k expert outputs of its assignments and sums them with
its gate weights.
"""
import numpy as np


def combine(y_perm, row_of_assign, topk_w, T: int, k: int):
    """out[t, :] = sum_{j<k} w[t, j] * y_perm[row_of_assign[t*k + j], :], j ascending, fp64."""
    y = np.asarray(y_perm, dtype=np.float64)
    w = np.asarray(topk_w, dtype=np.float64).reshape(T, k)
    rows = np.asarray(row_of_assign, dtype=np.int64).reshape(T, k)
    out = np.zeros((T, y.shape[1]), dtype=np.float64)
    for j in range(k):
        out += w[:, j:j + 1] * y[rows[:, j], :]
    return out
