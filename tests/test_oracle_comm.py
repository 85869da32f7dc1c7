"""Pins for the cross-rank traffic oracle (CPU)."""
import numpy as np
import pytest

from conftest import read_golden
from oracle import route_topk, histogram, plan_duplicates, permute, home_slot, skewness
from oracle.comm import comm_matrices, crossing_rows, max_inbound, owner_rank, segment_of_row
from paper_2506_07366_amd import workloads as wl

SMALL = wl.MoEConfig("small", T=300, d=16, ffn=8, E=12, k=3, G=4, S=5, dtype="f32", mode=1,
                     alpha=0.3, sigma_pred=0.3, acc=0.8, seed=5)


def run_case(cfg, pred_override=None):
    logits = wl.gen_logits(cfg)
    idx, _ = route_topk(logits, cfg.k)
    hist = histogram(idx, cfg.E)
    pred_idx = None
    if cfg.mode == 2:
        pred_idx = wl.gen_pred_idx(cfg, idx) if pred_override is None else pred_override(idx)
        hp = histogram(pred_idx, cfg.E)
    else:
        hp = wl.gen_pred_hist(cfg, hist)
    plan = plan_duplicates(cfg.mode, hp, cfg.E, cfg.G, cfg.S, cfg.cmax)
    x = np.zeros((cfg.T, 4))
    r = permute(cfg.mode, x, idx, pred_idx, hist, hp, plan.slot_expert, plan.slot_quota, cfg.E, cfg.G, cfg.S)
    disp, comb = comm_matrices(cfg.mode, idx, pred_idx, r["row_of_assign"], r["seg_offsets"], cfg.G, cfg.S)
    return idx, pred_idx, r, disp, comb


def test_figure2_scenario_by_hand():
    g = read_golden("comm_fig2.txt")
    T, G = int(g["T"][0]), int(g["G"][0])
    idx = np.array(g["topk_idx"], dtype=np.int64).reshape(T, 1)
    hist = histogram(idx, G)
    assert skewness(hist) == float(g["skewness"][0])
    plan = plan_duplicates(0, hist, G, G, 1, 1)
    r = permute(0, np.zeros((T, 2)), idx, None, hist, hist, plan.slot_expert, plan.slot_quota, G, G, 1)
    disp, comb = comm_matrices(0, idx, None, r["row_of_assign"], r["seg_offsets"], G, 1)
    want = np.array([g[f"dispatch_row{i}"] for i in range(G)], dtype=np.int64)
    assert np.array_equal(disp, want)
    assert np.array_equal(comb, want.T)
    assert crossing_rows(disp) == int(g["crossing_rows"][0])
    assert max_inbound(disp) == int(g["max_inbound"][0])
    # the paper's bottleneck expression
    assert max_inbound(disp) == (G - 1) * skewness(hist) / G**2 * T


@pytest.mark.parametrize("N,m", [(2, 4), (4, 8), (8, 16)])
def test_balanced_round_robin_moves_n_minus_1_over_n(N, m):
    # N ranks, one expert each, token t -> expert t mod N: every owner's m tokens spread
    # evenly, so (N-1)/N of them leave and every rank sends (N-1)/N^2 of all tokens
    T = N * m
    idx = (np.arange(T) % N).reshape(T, 1)
    hist = histogram(idx, N)
    plan = plan_duplicates(0, hist, N, N, 1, 1)
    r = permute(0, np.zeros((T, 2)), idx, None, hist, hist, plan.slot_expert, plan.slot_quota, N, N, 1)
    disp, comb = comm_matrices(0, idx, None, r["row_of_assign"], r["seg_offsets"], N, 1)
    assert crossing_rows(disp) * N == T * (N - 1)
    out = disp.sum(axis=1) - np.diag(disp)
    assert np.all(out * N * N == T * (N - 1))
    assert np.all(disp == m // N)


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_conservation_against_the_permutation(mode):
    cfg = SMALL.replace(mode=mode)
    idx, pred_idx, r, disp, comb = run_case(cfg)
    assert disp.sum() == cfg.A and comb.sum() == cfg.A
    # what arrives at a rank is its load; what it returns is the same rows
    assert np.array_equal(disp.sum(axis=0), r["rank_load"])
    assert np.array_equal(comb.sum(axis=1), r["rank_load"])
    owners = np.array([owner_rank(t, cfg.T, cfg.G) for t in range(cfg.T)])
    per_owner = np.bincount(owners, minlength=cfg.G) * cfg.k
    assert np.array_equal(comb.sum(axis=0), per_owner)
    if mode != 2:
        assert np.array_equal(disp.sum(axis=1), per_owner)
        assert np.array_equal(comb, disp.T)


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_vectorised_recount(mode):
    cfg = SMALL.replace(mode=mode)
    idx, pred_idx, r, disp, comb = run_case(cfg)
    a = np.arange(cfg.A)
    seg = np.searchsorted(np.asarray(r["seg_offsets"]), np.asarray(r["row_of_assign"]), side="right") - 1
    dst = seg // cfg.S
    own = ((a // cfg.k) * cfg.G) // cfg.T
    src = own.copy()
    if mode == 2:
        hit = (pred_idx[:, None, :] == idx[:, :, None]).any(axis=2).reshape(-1)
        src[hit] = dst[hit]
    d2 = np.zeros((cfg.G, cfg.G), dtype=np.int64)
    np.add.at(d2, (src, dst), 1)
    c2 = np.zeros((cfg.G, cfg.G), dtype=np.int64)
    np.add.at(c2, (dst, own), 1)
    assert np.array_equal(disp, d2) and np.array_equal(comb, c2)


def test_perfect_token_prediction_needs_no_dispatch():
    cfg = SMALL.replace(mode=2)
    idx, pred_idx, r, disp, comb = run_case(cfg, pred_override=lambda idx: idx.copy())
    assert crossing_rows(disp) == 0
    assert np.array_equal(np.diag(disp), r["rank_load"])


def test_all_mispredicted_goes_from_owner_to_home_rank():
    cfg = SMALL.replace(mode=2)
    # predicted ids disjoint from the true ones: shift every id by E/2 and fix collisions
    def wrong(idx):
        T, k = idx.shape
        out = np.empty_like(idx)
        for t in range(T):
            free = [e for e in range(cfg.E) if e not in set(idx[t].tolist())]
            out[t] = free[:k]
        return out
    idx, pred_idx, r, disp, comb = run_case(cfg, pred_override=wrong)
    H = -(-cfg.E // cfg.G)
    want = np.zeros((cfg.G, cfg.G), dtype=np.int64)
    for t in range(cfg.T):
        for j in range(cfg.k):
            want[owner_rank(t, cfg.T, cfg.G), home_slot(int(idx[t, j]), cfg.E, cfg.G, cfg.S) // cfg.S] += 1
    assert np.array_equal(disp, want)
    assert H >= 1


def test_duplication_lowers_the_bottleneck_inbound():
    # hot expert replicated across ranks: the busiest receiver gets fewer rows than at home
    cfg = SMALL.replace(mode=1, alpha=0.1, sigma_pred=0.0)
    _, _, _, disp1, _ = run_case(cfg)
    _, _, _, disp0, _ = run_case(cfg.replace(mode=0))
    assert disp1.sum(axis=0).max() <= disp0.sum(axis=0).max()


def test_segment_lookup_against_a_linear_scan():
    so = [0, 0, 3, 3, 3, 7, 8, 8]
    for row in range(8):
        want = [s for s in range(len(so) - 1) if so[s] <= row < so[s + 1]]
        assert len(want) == 1 and segment_of_row(row, so) == want[0]
    with pytest.raises(ValueError):
        segment_of_row(8, so)
    with pytest.raises(ValueError):
        segment_of_row(-1, so)


def test_pessimistic_errors_all_land_on_one_rank():
    # Section 3.3: with every misprediction on experts homed on rank 0, all dispatch transfers end there
    cfg = wl.MoEConfig("pess", T=1500, d=16, ffn=8, E=24, k=3, G=4, S=8, dtype="f32", mode=2, alpha=1.0,
                       acc=0.8, seed=13)
    on0 = np.array([home_slot(e, cfg.E, cfg.G, cfg.S) // cfg.S == 0 for e in range(cfg.E)])
    idx, pred_idx, r, disp, comb = run_case(cfg, pred_override=lambda i: wl.gen_pred_idx_concentrated(cfg, i, on0))
    wrong = (pred_idx != idx)
    assert wrong.sum() > 0 and np.all(on0[idx[wrong]])
    off = disp - np.diag(np.diag(disp))
    assert off[:, 1:].sum() == 0
    # each wrong entry costs one row into rank 0 unless its owner is rank 0 itself
    owners = (np.arange(cfg.T) * cfg.G) // cfg.T
    assert off[:, 0].sum() == int((wrong & (owners[:, None] != 0)).sum())
    assert r["rank_load"].argmax() == 0
