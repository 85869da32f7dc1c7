"""Oracle: rows that cross expert-parallel ranks (test infrastructure, CPU only).

Background, paragraph on the communication cost of routing: after the scatter a
rank holds a share of the tokens regardless of where their experts are, so with
N ranks and a balanced distribution a fraction (N-1)/N of every rank's rows
leaves it, and the rank of the most popular expert receives skewness times the
average.  The all-to-all after the FFN moves the same rows back.  Section 3.2.2:
with Token-to-Expert prediction a token is sent straight to the rank of its
predicted expert, so a correctly predicted assignment needs no transfer at
dispatch; a mispredicted one still has to reach the rank of its true expert
(Section 3.3: misrouted tokens always cost extra transfers).

Reading used here (the paper gives no placement rule for tokens): token t is
owned by rank floor(t*G/T) (contiguous equal shares of the batch).  Dispatch:
assignment (t, j) travels owner(t) -> rank of its segment, except that under
Token-to-Expert prediction an assignment whose true expert is among the token's
predicted experts is already in place (source = destination).  Combine: every
row's result travels rank of its segment -> owner(t).

Plain loops over the assignments, in the order a = t*k + j.
"""
import bisect

import numpy as np

from .plan import MODE_TOKEN


def owner_rank(t: int, T: int, G: int) -> int:
    return (t * G) // T


def segment_of_row(row: int, seg_offsets) -> int:
    """The segment sigma with seg_offsets[sigma] <= row < seg_offsets[sigma + 1]
    (seg_offsets is non-decreasing; empty segments have equal bounds)."""
    if not seg_offsets[0] <= row < seg_offsets[-1]:
        raise ValueError("row outside every segment")
    return bisect.bisect_right(seg_offsets, row) - 1


def comm_matrices(mode, topk_idx, pred_idx, row_of_assign, seg_offsets, G: int, S: int):
    """Returns (dispatch, combine), each int64 [G, G] with [source, destination] row counts."""
    idx = np.asarray(topk_idx, dtype=np.int64)
    T, k = idx.shape
    so = [int(v) for v in np.asarray(seg_offsets).reshape(-1)]
    rows = np.asarray(row_of_assign, dtype=np.int64).reshape(T, k)
    pred = None if pred_idx is None else np.asarray(pred_idx, dtype=np.int64).reshape(T, k)
    dispatch = np.zeros((G, G), dtype=np.int64)
    combine = np.zeros((G, G), dtype=np.int64)
    for t in range(T):
        own = owner_rank(t, T, G)
        for j in range(k):
            dst = segment_of_row(int(rows[t, j]), so) // S
            src = own
            if mode == MODE_TOKEN and any(int(idx[t, j]) == int(v) for v in pred[t]):
                src = dst
            dispatch[src, dst] += 1
            combine[dst, own] += 1
    return dispatch, combine


def crossing_rows(m) -> int:
    m = np.asarray(m)
    return int(m.sum() - np.trace(m))


def max_inbound(m) -> int:
    """Most rows any rank receives from the others."""
    m = np.asarray(m)
    return int((m.sum(axis=0) - np.diag(m)).max())
