"""Pins for the routing and histogram oracle (CPU)."""
import math

import numpy as np
import pytest
import torch

from conftest import read_golden
from oracle import route_topk, histogram, skewness, dist_error_rate
from paper_2506_07366_amd import workloads as wl


def brute_topk_row(row, k):
    """k rounds of 'take the largest remaining value, lowest index on ties'."""
    row = list(row)
    taken = []
    for _ in range(k):
        best = None
        for e, v in enumerate(row):
            if e in taken:
                continue
            if best is None or v > row[best]:
                best = e
        taken.append(best)
    return taken


@pytest.mark.parametrize("E,k", [(8, 2), (64, 6), (128, 8), (5, 5), (7, 1)])
def test_route_matches_brute_force_and_library(E, k):
    rng = np.random.default_rng(E * 100 + k)
    logits = rng.standard_normal((97, E)).astype(np.float32)
    idx, w = route_topk(logits, k)
    assert idx.dtype == np.int32 and idx.shape == (97, k)
    for t in range(97):
        assert list(idx[t]) == brute_topk_row(logits[t], k)
        assert len(set(idx[t])) == k
    # rows have distinct values, so a library top-k must agree exactly
    tv, ti = torch.topk(torch.from_numpy(logits), k, dim=1, largest=True, sorted=True)
    assert np.array_equal(ti.numpy(), idx)
    # softmax over the selected logits == library softmax
    ref = torch.softmax(tv.double(), dim=1).numpy()
    assert np.allclose(w, ref, rtol=0, atol=1e-15)
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-14)
    assert np.all(np.diff(w, axis=1) <= 0)          # descending logits -> descending weights


def test_route_tie_break_lowest_index():
    rng = np.random.default_rng(7)
    # logits quantised to multiples of 0.25: many exact ties
    logits = (np.round(rng.standard_normal((300, 16)) * 2) / 4).astype(np.float32)
    idx, w = route_topk(logits, 4)
    n_ties = 0
    for t in range(300):
        assert list(idx[t]) == brute_topk_row(logits[t], 4)
        vals = logits[t, idx[t]]
        for j in range(3):
            if vals[j] == vals[j + 1]:
                n_ties += 1
                assert idx[t, j] < idx[t, j + 1]
    assert n_ties > 50
    # an all-equal row picks experts 0..k-1 with equal weights
    idx, w = route_topk(np.zeros((1, 9), np.float32), 3)
    assert list(idx[0]) == [0, 1, 2] and np.allclose(w, 1 / 3)


def test_route_k1_weight_is_one_and_closed_form():
    logits = np.array([[0.0, math.log(3.0), -1.0]], dtype=np.float64)
    idx, w = route_topk(logits, 1)
    assert list(idx[0]) == [1] and w[0, 0] == 1.0
    idx, w = route_topk(logits, 2)
    # softmax over {log 3, 0} = {3/4, 1/4}
    assert list(idx[0]) == [1, 0]
    assert np.allclose(w[0], [0.75, 0.25], atol=1e-15)


def test_histogram_pins():
    rng = np.random.default_rng(3)
    idx = rng.integers(0, 13, size=(500, 4)).astype(np.int32)
    h = histogram(idx, 13)
    assert h.dtype == np.int32
    assert np.array_equal(h, np.bincount(idx.reshape(-1), minlength=13))
    assert h.sum() == idx.size                     # sums to T*k
    assert np.array_equal(histogram(np.zeros((0, 2), np.int32), 4), np.zeros(4, np.int32))
    # position of the count matters (catches an off-by-one in the bin index)
    assert list(histogram(np.array([2, 2, 0]), 4)) == [1, 0, 2, 0]


def test_skewness_paper_value():
    g = read_golden("skewness_fig2.txt")
    assert skewness(np.array(g["hist"])) == pytest.approx(g["skewness"][0], abs=1e-12)
    assert skewness(np.array([5, 5, 5, 5])) == 1.0


def test_dist_error_rate_closed_form():
    # p_hat = (.5,.5), p = (.75,.25): |diff| = .25 each, mean .25, / (1/2) = 0.5
    assert dist_error_rate([50, 50], [75, 25]) == pytest.approx(0.5)
    assert dist_error_rate([3, 1, 4], [3, 1, 4]) == 0.0


def test_generated_routing_has_paper_like_skew():
    """The synthetic stand-in for the paper's routing traces is skewed at least as
    much as its datasets (Table 1: 1.39 - 1.99)."""
    cfg = wl.CONFIGS["cfg2_mixtral_dist"]
    idx, _ = route_topk(wl.gen_logits(cfg), cfg.k)
    h = histogram(idx, cfg.E)
    assert h.sum() == cfg.A
    assert skewness(h) > 1.3
    hp = wl.gen_pred_hist(cfg, h)
    assert hp.sum() == cfg.A and hp.min() >= 0
    assert 0.0 < dist_error_rate(hp, h) < 1.0
