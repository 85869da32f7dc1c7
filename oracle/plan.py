"""Oracle: the expert-duplication planner (test infrastructure, CPU only).

Algorithm 1 ("Expert Duplication in MoE Load Balancing", Section 3.1) in a
count-based form.  The paper's algorithm works on individual tokens; since all
tokens of one expert are interchangeable for load purposes, the state kept here
is, per rank g and slot s, which expert the slot hosts and how many of that
expert's tokens it is planned to serve.  A literal per-token version lives in
``alg1_literal.py`` and the tests check that both give the same per-(expert,
rank) loads.

Units and readings where the paper is silent or garbled:
  * per-GPU memory M and params(e) <= M_g become "S expert slots per rank, all
    experts the same size";
  * the initial placement is the home placement: H = ceil(E/G) experts per rank,
    expert e on rank e // H, slot e % H;
  * with top-k routing each (token, expert) assignment is one unit of load;
  * the printed algorithm reassigns tokens to g_c even when the replication test
    failed, i.e. to a GPU that does not host the expert.  Here tokens move only
    to a rank that hosts the expert after the conditional copy;
  * when the paper's own candidate (coldest rank, hottest expert of the hottest
    rank) is infeasible the search continues: next experts of the hottest rank
    in descending load, then the next-coldest rank; the loop stops when nothing
    is feasible.  The first candidate tried is exactly the paper's;
  * the number moved is min(Delta, tokens of e* on g_h);
  * all arg-max / arg-min ties go to the lowest index;
  * the loop is capped at 16*G*S iterations (it terminates anyway: each move
    strictly lowers the sum of squared rank loads).
"""
from dataclasses import dataclass

import numpy as np

MODE_NONE = 0
MODE_DISTRIBUTION = 1
MODE_TOKEN = 2


@dataclass
class Plan:
    slot_expert: np.ndarray     # [G*S] int32, -1 = empty slot
    slot_quota: np.ndarray      # [G*S] int32, planned rows per slot
    rank_load_pred: np.ndarray  # [G] int32, planned rows per rank
    n_iters: int


def home_slot(e: int, E: int, G: int, S: int) -> int:
    """Global slot id (g*S + s) of expert e's home."""
    H = -(-E // G)
    return (e // H) * S + (e % H)


def plan_duplicates(mode: int, hist_pred, E: int, G: int, S: int, c_max: int) -> Plan:
    """Build the slot table and per-slot planned quotas from predicted counts.

    mode 0 stops after the home placement; modes 1 and 2 run the greedy loop of
    Algorithm 1 (for mode 2 the caller passes the histogram of the predicted
    per-token ids)."""
    H = -(-E // G)
    assert H <= S, "every expert needs a home slot"
    n_hat = [int(v) for v in np.asarray(hist_pred).reshape(-1)]
    assert len(n_hat) == E and min(n_hat) >= 0

    slot_expert = [[-1] * S for _ in range(G)]
    quota = [[0] * S for _ in range(G)]
    copies = [1] * E
    # initial dispatch: every token goes to the only rank hosting its expert
    for e in range(E):
        slot_expert[e // H][e % H] = e
        quota[e // H][e % H] = n_hat[e]
    L = [sum(quota[g]) for g in range(G)]

    n_iters = 0
    if mode != MODE_NONE:
        i_max = 16 * G * S
        while n_iters < i_max:
            g_h = max(range(G), key=lambda g: (L[g], -g))          # hottest, ties -> lowest g
            if L[g_h] - min(L) <= 1:                               # loop guard of Algorithm 1
                break
            cold_order = sorted((g for g in range(G) if g != g_h), key=lambda g: (L[g], g))
            hot_slots = sorted((s for s in range(S) if quota[g_h][s] > 0),
                               key=lambda s: (-quota[g_h][s], s))  # e* first
            move = None
            for g_c in cold_order:
                if L[g_h] - L[g_c] <= 1:
                    break
                for s in hot_slots:
                    e = slot_expert[g_h][s]
                    hosting = [sp for sp in range(S) if slot_expert[g_c][sp] == e]
                    if hosting:
                        move = (g_c, s, hosting[0], False)
                        break
                    empty = [sp for sp in range(S) if slot_expert[g_c][sp] == -1]
                    if copies[e] < c_max and empty:
                        move = (g_c, s, empty[0], True)
                        break
                if move is not None:
                    break
            if move is None:
                break
            g_c, s, sp, new_replica = move
            e = slot_expert[g_h][s]
            if new_replica:                                        # copy weights of e* on g_c
                slot_expert[g_c][sp] = e
                copies[e] += 1
            delta = -(-(L[g_h] - L[g_c]) // 2)                     # ceil((L_h - L_c) / 2)
            m = min(delta, quota[g_h][s])
            quota[g_h][s] -= m
            quota[g_c][sp] += m
            L[g_h] -= m
            L[g_c] += m
            n_iters += 1

    return Plan(
        slot_expert=np.array(slot_expert, dtype=np.int32).reshape(-1),
        slot_quota=np.array(quota, dtype=np.int32).reshape(-1),
        rank_load_pred=np.array(L, dtype=np.int32),
        n_iters=n_iters,
    )
