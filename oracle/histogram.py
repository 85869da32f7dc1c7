"""Oracle: per-expert token counts and the imbalance metrics built on them
(test infrastructure, CPU only)."""
import numpy as np


def histogram(idx: np.ndarray, E: int) -> np.ndarray:
    """n_e = number of assignments routed to expert e (the n_i of Eq. (1); the
    quantity Distribution-Only Prediction forecasts as p_hat_i = n_i / N)."""
    n = np.zeros(E, dtype=np.int64)
    for e in np.asarray(idx).reshape(-1):
        n[int(e)] += 1
    return n.astype(np.int32)


def skewness(hist: np.ndarray) -> float:
    """Tokens on the most popular expert divided by the average tokens per expert
    ("Quantifying Imbalance", Background).  With top-k routing every (token,
    expert) assignment counts as one token."""
    hist = np.asarray(hist, dtype=np.float64)
    return float(hist.max() / (hist.sum() / hist.size))


def dist_error_rate(hist_pred: np.ndarray, hist_true: np.ndarray) -> float:
    """Distribution-Only error rate |p_hat - p| / (1 / #experts), averaged over
    experts (Section 3.2.1; "averaged L1 distance over number of experts",
    Section 3.3)."""
    hp = np.asarray(hist_pred, dtype=np.float64)
    ht = np.asarray(hist_true, dtype=np.float64)
    E = hp.size
    return float(np.mean(np.abs(hp / hp.sum() - ht / ht.sum())) / (1.0 / E))
