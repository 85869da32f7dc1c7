"""Pins for the Distribution-Only predictor oracle (CPU)."""
from fractions import Fraction

import numpy as np
import pytest

from oracle.predictor import predictor_update, predictor_estimate, predictor_predict
from oracle import dist_error_rate


def test_hand_cases():
    # three equal experts, 10 assignments: 3 each, the spare one goes to the lowest index
    assert predictor_predict([3, 3, 3], 10) == [4, 3, 3]
    # 75 % on one of four experts (the Figure 2 distribution), 8 assignments, worked by hand: p = (.75, 1/12, 1/12, 1/12) * 8 = (6, 2/3, 2/3, 2/3): floors 6 0 0 0, two spare -> e1, e2
    assert predictor_predict([900, 100, 100, 100], 8) == [6, 1, 1, 0]
    # nothing seen yet: uniform
    assert predictor_predict([0, 0, 0, 0], 6) == [2, 2, 1, 1]
    assert predictor_predict([5, 0], 0) == [0, 0]
    assert predictor_update([1, 2, 3], [10, 0, 5]) == [11, 2, 8]


@pytest.mark.parametrize("seed", range(5))
def test_sum_and_quota_property(seed):
    rng = np.random.default_rng(seed)
    E = int(rng.integers(1, 200))
    counts = [int(v) for v in rng.integers(0, 10**9, size=E)]
    A = int(rng.integers(0, 2**31 - 1))
    pred = predictor_predict(counts, A)
    assert sum(pred) == A
    num, den = predictor_estimate(counts)
    for e in range(E):
        exact = Fraction(num[e] * A, den)
        assert abs(Fraction(pred[e]) - exact) < 1       # largest remainder stays within one of the quota
        assert pred[e] >= 0


def test_estimate_maximises_the_multinomial_likelihood():
    # Appendix A: among all distributions on the simplex, n / N maximises sum n_i log p_i
    rng = np.random.default_rng(3)
    n = rng.integers(1, 50, size=6)
    num, den = predictor_estimate(n.tolist())
    p_hat = np.array(num, dtype=np.float64) / den
    best = float(np.sum(n * np.log(p_hat)))
    for _ in range(2000):
        q = rng.dirichlet(np.ones(6))
        assert float(np.sum(n * np.log(q))) <= best + 1e-12
    for _ in range(200):      # small moves around the estimate
        q = p_hat + rng.normal(0, 1e-3, size=6)
        q = np.abs(q) / np.abs(q).sum()
        assert float(np.sum(n * np.log(q))) <= best + 1e-12


def test_batches_give_the_running_average():
    rng = np.random.default_rng(4)
    p = rng.dirichlet(np.full(16, 0.3))
    counts = [0] * 16
    per_batch, sizes = [], []
    for b in range(12):
        N_b = int(rng.integers(100, 5000))
        h = rng.multinomial(N_b, p)
        per_batch.append(h / N_b)
        sizes.append(N_b)
        counts = predictor_update(counts, h.tolist())
        num, den = predictor_estimate(counts)
        want = np.average(np.array(per_batch), axis=0, weights=np.array(sizes, dtype=np.float64))
        assert den == sum(sizes)
        assert np.allclose(np.array(num) / den, want, rtol=0, atol=1e-12)


def test_error_rate_shrinks_with_the_data_seen():
    # i.i.d. draws: |p_hat - p| falls like 1/sqrt(N), so 100x the tokens give about a tenth of the error
    rng = np.random.default_rng(5)
    E = 8
    p = rng.dirichlet(np.full(E, 0.5))
    errs = []
    for N in (2000, 200000):
        e = []
        for _ in range(20):
            h = rng.multinomial(N, p)
            pred = predictor_predict(h.tolist(), 10**6)
            e.append(dist_error_rate(np.array(pred), p * 10**6))
        errs.append(np.mean(e))
    assert errs[1] < errs[0] / 5
    assert errs[1] < 0.02


def test_predicting_the_seen_total_returns_the_counts():
    rng = np.random.default_rng(6)
    counts = [int(v) for v in rng.integers(0, 1000, size=64)]
    assert predictor_predict(counts, sum(counts)) == counts
