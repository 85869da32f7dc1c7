"""Pins for the dispatch / permutation oracle (CPU)."""
import numpy as np
import pytest

from conftest import read_golden
from oracle import route_topk, histogram, plan_duplicates, permute, home_slot, skewness
from paper_2506_07366_amd import workloads as wl


def make_case(cfg):
    logits = wl.gen_logits(cfg)
    idx, w = route_topk(logits, cfg.k)
    hist = histogram(idx, cfg.E)
    pred_idx = None
    if cfg.mode == 2:
        pred_idx = wl.gen_pred_idx(cfg, idx)
        hp = histogram(pred_idx, cfg.E)
    else:
        hp = wl.gen_pred_hist(cfg, hist)
    plan = plan_duplicates(cfg.mode, hp, cfg.E, cfg.G, cfg.S, cfg.cmax)
    return idx, w, hist, hp, pred_idx, plan


SMALL = wl.MoEConfig("small", T=300, d=16, ffn=8, E=12, k=3, G=4, S=5, dtype="f32", mode=1,
                     alpha=0.3, sigma_pred=0.3, acc=0.8, seed=5)


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_permutation_invariants(mode):
    cfg = SMALL.replace(mode=mode)
    idx, w, hist, hp, pred_idx, plan = make_case(cfg)
    x = wl.gen_x(cfg)
    r = permute(mode, x, idx, pred_idx, hist, hp, plan.slot_expert, plan.slot_quota, cfg.E, cfg.G, cfg.S)
    A = cfg.A
    # bijection on [0, A)
    assert sorted(r["row_of_assign"].tolist()) == list(range(A))
    assert np.array_equal(r["assign_of_row"][r["row_of_assign"]], np.arange(A))
    flat = idx.reshape(-1)
    so = r["seg_offsets"]
    assert so[0] == 0 and so[-1] == A and np.all(np.diff(so) >= 0)
    for s in range(cfg.nseg):
        rows = r["assign_of_row"][so[s]:so[s + 1]]
        # every row of a segment is served by the expert that slot hosts
        assert np.all(flat[rows] == plan.slot_expert[s])
        assert np.all(np.diff(rows) > 0)                 # stable: ascending a
    assert r["rank_load"].sum() == A
    # rows are byte-equal to their source token rows
    assert np.array_equal(r["x_perm"], x[r["assign_of_row"] // cfg.k])
    # a library stable sort by (segment, a) gives the same permutation
    order = np.argsort(r["seg"], kind="stable")
    assert np.array_equal(order, r["assign_of_row"])


def test_mode0_bottleneck_equals_hottest_expert():
    g = read_golden("skewness_fig2.txt")
    n = g["hist"]
    idx = np.repeat(np.arange(4), n).astype(np.int32)[:, None]
    rng = np.random.default_rng(0)
    rng.shuffle(idx)
    plan = plan_duplicates(0, n, 4, 4, 2, 4)
    r = permute(0, None, idx, None, n, n, plan.slot_expert, plan.slot_quota, 4, 4, 2)
    assert r["rank_load"].max() == g["max_rank_load_mode0"][0]
    assert r["rank_load"].max() == pytest.approx(skewness(np.array(n)) * sum(n) / 4)


def test_mode1_exact_prediction_reproduces_planned_loads():
    cfg = SMALL.replace(mode=1, sigma_pred=0.0)
    idx, w, hist, hp, pred_idx, plan = make_case(cfg)
    assert np.array_equal(hp, hist)
    r = permute(1, None, idx, None, hist, hp, plan.slot_expert, plan.slot_quota, cfg.E, cfg.G, cfg.S)
    assert np.array_equal(np.diff(r["seg_offsets"]), plan.slot_quota)
    assert np.array_equal(r["rank_load"], plan.rank_load_pred)


def test_mode1_proportional_split_hand_case():
    # one expert, n = 10 true rows, predicted 20 split 10 | 6 | 4 over three replicas:
    # boundaries floor(10*{0,10,16,20}/20) = 0,5,8,10 -> 5,3,2 rows
    E, G, S = 1, 3, 1
    idx = np.zeros((10, 1), np.int32)
    r = permute(1, None, idx, None, [10], [20], [0, 0, 0], [10, 6, 4], E, G, S)
    assert list(np.diff(r["seg_offsets"])) == [5, 3, 2]
    assert list(r["seg"]) == [0] * 5 + [1] * 3 + [2] * 2
    # zero predicted count -> home slot
    r = permute(1, None, idx, None, [10], [0], [0, -1, -1], [0, 0, 0], E, G, S)
    assert list(np.diff(r["seg_offsets"])) == [10, 0, 0]


def test_mode2_fallback_rows_counted_independently():
    cfg = SMALL.replace(mode=2)
    idx, w, hist, hp, pred_idx, plan = make_case(cfg)
    r = permute(2, None, idx, pred_idx, hist, hp, plan.slot_expert, plan.slot_quota, cfg.E, cfg.G, cfg.S)
    miss = 0
    hit_per_slot = np.zeros(cfg.nseg, dtype=np.int64)
    for t in range(cfg.T):
        for j in range(cfg.k):
            if idx[t, j] not in set(pred_idx[t].tolist()):
                miss += 1
                assert r["seg"][t * cfg.k + j] == home_slot(int(idx[t, j]), cfg.E, cfg.G, cfg.S)
            else:
                hit_per_slot[r["seg"][t * cfg.k + j]] += 1
    assert 0 < miss < cfg.A
    # correctly predicted rows never exceed the planned quota of their slot
    assert np.all(hit_per_slot <= plan.slot_quota)
    # perfect prediction: every slot gets exactly its quota
    cfg = SMALL.replace(mode=2, acc=1.0)
    idx, w, hist, hp, pred_idx, plan = make_case(cfg)
    assert np.array_equal(pred_idx, idx)
    r = permute(2, None, idx, pred_idx, hist, hp, plan.slot_expert, plan.slot_quota, cfg.E, cfg.G, cfg.S)
    assert np.array_equal(np.diff(r["seg_offsets"]), plan.slot_quota)


def test_mode2_hand_case():
    # E=2, G=2, S=2, k=1.  Predicted ids: t0..t3 -> e0, t4 -> e1.  Plan splits e0 2|2.
    # True ids: t0,t1,t2 -> e0 (hits, pred ranks 0,1,2), t3 -> e1 (miss -> home of e1), t4 -> e1 (hit)
    idx = np.array([[0], [0], [0], [1], [1]], np.int32)
    pred = np.array([[0], [0], [0], [0], [1]], np.int32)
    slot_expert = [0, -1, 1, 0]
    slot_quota = [2, 0, 1, 2]
    r = permute(2, None, idx, pred, [3, 2], [4, 1], slot_expert, slot_quota, 2, 2, 2)
    assert list(r["seg"]) == [0, 0, 3, 2, 2]
    assert list(r["seg_offsets"]) == [0, 2, 2, 4, 5]
    assert list(r["row_of_assign"]) == [0, 1, 4, 2, 3]
    assert list(r["rank_load"]) == [2, 3]


def test_empty_input():
    r = permute(0, np.zeros((0, 4), np.float32), np.zeros((0, 2), np.int32), None, [0, 0], [0, 0],
                [0, 1], [0, 0], 2, 2, 1)
    assert list(r["seg_offsets"]) == [0, 0, 0] and r["x_perm"].shape == (0, 4)
