"""Oracle cross-check: Algorithm 1 of Section 3.1 run token by token
(test infrastructure, CPU only; meant for tiny inputs).

The state is the paper's: every token has an expert (the map f) and a GPU it is
dispatched to (d); the placement says which GPUs hold a copy of which expert; L_g
counts the tokens dispatched to GPU g.  Nothing is aggregated into per-slot
quotas as in ``plan.py``: loads are recounted from d at every iteration and
tokens are re-dispatched one by one, so the two forms share only the readings
of the paper listed in ``plan.py`` (tokens move only to a GPU that holds the
expert; when the hottest expert cannot go to the coldest GPU the search goes on
with the next experts and then the next-coldest GPUs; memory is S equal slots).

Experts that serve equally many tokens on the hot GPU are taken in the order of
the slots they occupy there: the home experts of a GPU sit in its first slots by
ascending id, a copy takes the lowest free slot when it is made and is never
removed.  The placement is therefore kept as a slot list per GPU.
"""
import numpy as np


def alg1_literal(f, E: int, G: int, S: int, c_max: int, max_iters=None):
    """Returns (load[e][g] = tokens of expert e dispatched to GPU g, P, d, n_iters);
    P is the placement as a set of (expert, GPU) pairs."""
    f = [int(v) for v in f]
    T = len(f)
    H = -(-E // G)
    slots = [[None] * S for _ in range(G)]               # slots[g][s] = expert held there
    for e in range(E):
        slots[e // H][e % H] = e                         # initial (home) placement

    def holds(g, e):
        return e in slots[g]

    # Initial dispatch: each token goes to the lowest-numbered GPU that holds its expert.
    d = [min(g for g in range(G) if holds(g, f[t])) for t in range(T)]
    n_iters = 0
    if max_iters is None:
        max_iters = 16 * G * S
    while n_iters < max_iters:
        L = [d.count(g) for g in range(G)]
        if max(L) - min(L) <= 1:                         # balanced: nothing left to do
            break
        hot = max(range(G), key=lambda g: (L[g], -g))
        moved = False
        for cold in sorted((g for g in range(G) if g != hot), key=lambda g: (L[g], g)):
            gap = L[hot] - L[cold]
            if gap <= 1:
                break
            half_gap = -(-gap // 2)                      # tokens to shift: half the gap, rounded up
            served = {}                                  # tokens per expert on the hot GPU
            for t in range(T):
                if d[t] == hot:
                    served[f[t]] = served.get(f[t], 0) + 1
            # busiest expert first; equal counts in slot order on the hot GPU
            for e in sorted(served, key=lambda e: (-served[e], slots[hot].index(e))):
                if not holds(cold, e):
                    n_copies = sum(1 for g in range(G) if holds(g, e))
                    if n_copies < c_max and None in slots[cold]:
                        slots[cold][slots[cold].index(None)] = e   # a new copy of e on the cold GPU
                if holds(cold, e):
                    shifted = 0
                    for t in range(T):                   # the earliest tokens of e on the hot GPU
                        if shifted == half_gap:
                            break
                        if d[t] == hot and f[t] == e:
                            d[t] = cold
                            shifted += 1
                    moved = True
                    break
            if moved:
                break
        if not moved:
            break
        n_iters += 1
    load = np.zeros((E, G), dtype=np.int64)
    for t in range(T):
        load[f[t], d[t]] += 1
    P = {(e, g) for g in range(G) for e in slots[g] if e is not None}
    return load, P, d, n_iters
