"""Oracle: the Distribution-Only predictor (test infrastructure, CPU only).

Section 3.2.1, Eq. (1) and Appendix A: expert selection in a layer is modelled as
i.i.d. draws from a multinomial distribution, whose maximum-likelihood estimate is
p_hat_i = n_i / N with n_i the tokens that activated expert i among the N seen;
with data arriving in batches the estimate is the running average over all batches
seen so far.  The predicted histogram for a coming batch of A assignments is
p_hat * A brought to integers that sum to A by largest remainder (ties -> lowest
expert), the same rounding the seeded input generator uses.

Reading where the paper is silent: before any batch has been seen (N = 0) the
estimate is uniform.

Exact integer arithmetic on Python ints.
"""


def predictor_update(counts, hist):
    """Cumulative per-expert counts after one more batch."""
    if len(counts) != len(hist):
        raise ValueError("length mismatch")
    return [int(c) + int(h) for c, h in zip(counts, hist)]


def predictor_estimate(counts):
    """(numerators, denominator) of p_hat: n_i / N, uniform when nothing has been seen."""
    n = [int(c) for c in counts]
    N = sum(n)
    if N == 0:
        return [1] * len(n), len(n)
    return n, N


def predictor_predict(counts, A_next: int):
    """Predicted histogram for a batch of A_next assignments: floor(p_hat_i * A) plus one
    for the experts with the largest remainders, until the sum is A."""
    num, den = predictor_estimate(counts)
    A = int(A_next)
    base = [(c * A) // den for c in num]
    rem = [(c * A) % den for c in num]
    deficit = A - sum(base)
    order = sorted(range(len(num)), key=lambda e: (-rem[e], e))
    for e in order[:deficit]:
        base[e] += 1
    return base
