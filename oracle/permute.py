"""Oracle: dispatch of assignments to replicas and the token permutation
(test infrastructure, CPU only).

This stands where the all-to-all dispatch of expert parallelism is (Background,
paragraph on the communication cost of routing) and realises the dispatch d of
Algorithm 1 for a given plan.  An *assignment* is a = t*k + j: token t's j-th
selected expert.  A *segment* is one slot (g, s) of the plan, global id g*S + s;
the rows of a segment are the assignments that slot serves.

Readings where the paper is silent:
  * Algorithm 1 moves "the first Delta tokens" of an expert; after several moves
    the literal token->replica map depends on the order of moves.  Here replicas
    of an expert, in ascending slot id, take contiguous ranges of that expert's
    assignments in ascending a.  Loads and outputs are unaffected (replicas hold
    identical weights).
  * Distribution-Only: true counts follow a predicted split proportionally,
    range boundaries B_r = floor(n_e * Q_r / n_hat_e) with Q_r the cumulative
    planned quotas; n_hat_e = 0 sends everything to the home slot.
  * Token-to-Expert: a token is dispatched by its predicted ids; an assignment
    whose true expert is among the token's predicted ids takes its place in the
    plan (which was built from the histogram of the predicted ids); any other
    assignment falls back to the home slot of its true expert (the extra
    transfer of mispredicted tokens, Section 3.3).
"""
import numpy as np

from .plan import MODE_NONE, MODE_DISTRIBUTION, MODE_TOKEN, home_slot


def _replicas(slot_expert, E):
    """Per expert, its slots in ascending global slot id."""
    reps = [[] for _ in range(E)]
    for sigma, e in enumerate(slot_expert):
        if e >= 0:
            reps[int(e)].append(sigma)
    return reps


def dispatch_segments(mode, topk_idx, pred_idx, hist_true, hist_pred,
                      slot_expert, slot_quota, E, G, S):
    """Segment id for every assignment, int32 [A]."""
    idx = np.asarray(topk_idx, dtype=np.int64)
    T, k = idx.shape
    A = T * k
    flat = idx.reshape(-1)
    slot_expert = [int(v) for v in slot_expert]
    slot_quota = [int(v) for v in slot_quota]
    seg = np.empty(A, dtype=np.int32)

    if mode == MODE_NONE:
        for a in range(A):
            seg[a] = home_slot(int(flat[a]), E, G, S)
        return seg

    reps = _replicas(slot_expert, E)
    # cumulative planned quotas Q_0 = 0 <= ... <= Q_R per expert
    Q = []
    for e in range(E):
        q = [0]
        for sigma in reps[e]:
            q.append(q[-1] + slot_quota[sigma])
        Q.append(q)

    if mode == MODE_DISTRIBUTION:
        n = [int(v) for v in hist_true]
        n_hat = [int(v) for v in hist_pred]
        # range boundaries B_r = floor(n_e * Q_r / n_hat_e), exact integers
        B = [[(n[e] * q) // n_hat[e] for q in Q[e]] if n_hat[e] > 0 else None for e in range(E)]
        seen = [0] * E
        for a in range(A):
            e = int(flat[a])
            i = seen[e]
            seen[e] += 1
            if n_hat[e] == 0:
                seg[a] = home_slot(e, E, G, S)
                continue
            assert Q[e][-1] == n_hat[e]
            r = max(r for r in range(len(reps[e])) if B[e][r] <= i)
            assert B[e][r] <= i < B[e][r + 1]
            seg[a] = reps[e][r]
        return seg

    if mode == MODE_TOKEN:
        pred = np.asarray(pred_idx, dtype=np.int64).reshape(T, k)
        # stable rank of every predicted assignment among those of the same expert
        seen = [0] * E
        pred_rank = np.empty((T, k), dtype=np.int64)
        for t in range(T):
            for j in range(k):
                e = int(pred[t, j])
                pred_rank[t, j] = seen[e]
                seen[e] += 1
        for t in range(T):
            row = [int(v) for v in pred[t]]
            for j in range(k):
                e = int(idx[t, j])
                a = t * k + j
                if e in row:
                    jp = row.index(e)
                    i = int(pred_rank[t, jp])
                    r = max(r for r in range(len(reps[e])) if Q[e][r] <= i)
                    assert Q[e][r] <= i < Q[e][r + 1]
                    seg[a] = reps[e][r]
                else:
                    seg[a] = home_slot(e, E, G, S)
        return seg

    raise ValueError(mode)


def permute(mode, x, topk_idx, pred_idx, hist_true, hist_pred,
            slot_expert, slot_quota, E, G, S):
    """Stable counting sort of the assignments by segment and the row gather.

    Returns dict with seg (per assignment), seg_offsets [G*S+1], row_of_assign [A],
    assign_of_row [A], x_perm [A, d] (or None when x is None), rank_load [G]."""
    idx = np.asarray(topk_idx)
    T, k = idx.shape
    A = T * k
    nseg = G * S
    seg = dispatch_segments(mode, topk_idx, pred_idx, hist_true, hist_pred,
                            slot_expert, slot_quota, E, G, S)
    counts = [0] * nseg
    for a in range(A):
        counts[int(seg[a])] += 1
    seg_offsets = np.zeros(nseg + 1, dtype=np.int32)
    for s in range(nseg):
        seg_offsets[s + 1] = seg_offsets[s] + counts[s]
    fill = [int(v) for v in seg_offsets[:-1]]
    row_of_assign = np.empty(A, dtype=np.int32)
    assign_of_row = np.empty(A, dtype=np.int32)
    for a in range(A):                       # ascending a => stable within a segment
        s = int(seg[a])
        row_of_assign[a] = fill[s]
        assign_of_row[fill[s]] = a
        fill[s] += 1
    x_perm = None
    if x is not None:
        x = np.asarray(x)
        x_perm = x[assign_of_row // k, :].copy()
    rank_load = np.array([int(seg_offsets[(g + 1) * S] - seg_offsets[g * S]) for g in range(G)],
                         dtype=np.int32)
    return dict(seg=seg, seg_offsets=seg_offsets, row_of_assign=row_of_assign,
                assign_of_row=assign_of_row, x_perm=x_perm, rank_load=rank_load)
