"""Oracle cross-check: Algorithm 1 of Section 3.1 run token by token
(test infrastructure, CPU only; meant for tiny inputs).

State is exactly the paper's: a token->expert map f, a placement set P of
(expert, GPU) pairs, a dispatch d: token -> GPU and the per-GPU loads L.  The
same readings as in ``plan.py`` apply (tokens only move to a GPU that hosts the
expert; fall through to the next expert / next-coldest GPU when the first
candidate is infeasible; memory = S equally sized expert slots per GPU).
"""
import numpy as np


def alg1_literal(f, E: int, G: int, S: int, c_max: int, max_iters=None):
    """Returns (load[e][g] = tokens of expert e dispatched to GPU g, P, d, n_iters)."""
    f = [int(v) for v in f]
    T = len(f)
    H = -(-E // G)
    P = {(e, e // H) for e in range(E)}                  # initial placement
    # d(t) <- min{ g | (f(t), g) in P }
    d = [min(g for (e, g) in P if e == f[t]) for t in range(T)]
    n_iters = 0
    if max_iters is None:
        max_iters = 16 * G * S
    while n_iters < max_iters:
        L = [sum(1 for t in range(T) if d[t] == g) for g in range(G)]
        if max(L) - min(L) <= 1:
            break
        g_h = max(range(G), key=lambda g: (L[g], -g))
        done = False
        for g_c in sorted((g for g in range(G) if g != g_h), key=lambda g: (L[g], g)):
            if L[g_h] - L[g_c] <= 1:
                break
            delta = -(-(L[g_h] - L[g_c]) // 2)
            on_hot = {}
            for t in range(T):
                if d[t] == g_h:
                    on_hot[f[t]] = on_hot.get(f[t], 0) + 1
            # experts on g_h by tokens served there (descending); ties by the slot
            # order of the count-based form: home experts of g_h first (ascending
            # e), then replicas in the order they were created.  For tiny test
            # inputs ties are avoided by construction; ascending e is used here.
            for e in sorted(on_hot, key=lambda e: (-on_hot[e], e)):
                if (e, g_c) not in P:
                    copies = sum(1 for (ee, _) in P if ee == e)
                    hosted = sum(1 for (_, gg) in P if gg == g_c)
                    if copies < c_max and hosted < S:
                        P.add((e, g_c))                  # copy weights of e* on g_c
                if (e, g_c) in P:
                    movers = [t for t in range(T) if d[t] == g_h and f[t] == e][:delta]
                    for t in movers:                      # the first Delta tokens
                        d[t] = g_c
                    done = True
                    break
            if done:
                break
        if not done:
            break
        n_iters += 1
    load = np.zeros((E, G), dtype=np.int64)
    for t in range(T):
        load[f[t], d[t]] += 1
    return load, P, d, n_iters
