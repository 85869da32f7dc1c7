"""Oracle: exhaustive replica assignment on tiny E / G (test infrastructure, CPU only).

Quality bound for the greedy planner of Algorithm 1: the best achievable
max-rank load (Section 3.1 states the goal: every GPU ends up with the same
number of tokens) over every way of filling the spare slots with replicas.

For a fixed placement the tokens of an expert may be split freely over the
ranks that host it, so the smallest feasible max-rank load M is the smallest M
for which a flow experts -> hosting ranks with rank capacity M carries all
tokens.  By the max-flow / min-cut (Hall) condition that is
    max over non-empty expert sets X of ceil( sum_{e in X} n_e / |ranks hosting some e in X| ).
"""
import itertools


def best_split_makespan(n, hosts, G):
    """Min over token splits of the max rank load, for a fixed placement.
    hosts[e] = set of ranks hosting expert e."""
    E = len(n)
    best = 0
    for mask in range(1, 1 << E):
        tot = 0
        ranks = set()
        for e in range(E):
            if mask >> e & 1:
                tot += n[e]
                ranks |= hosts[e]
        if tot > 0:
            best = max(best, -(-tot // len(ranks)))
    return best


def optimal_makespan(n, G, S, c_max):
    """Min over all placements (home slots fixed, every spare slot empty or
    holding any expert, at most c_max copies per expert) of the best split."""
    n = [int(v) for v in n]
    E = len(n)
    H = -(-E // G)
    home_rank = [e // H for e in range(E)]
    spare = []                                   # rank of every spare slot
    for g in range(G):
        homes = sum(1 for e in range(E) if home_rank[e] == g)
        spare += [g] * (S - homes)
    best = None
    for fill in itertools.product(range(-1, E), repeat=len(spare)):
        hosts = [{home_rank[e]} for e in range(E)]
        for g, e in zip(spare, fill):
            if e >= 0:
                hosts[e].add(g)
        if any(len(hosts[e]) > c_max for e in range(E)):
            continue
        m = best_split_makespan(n, hosts, G)
        if best is None or m < best:
            best = m
    return best
