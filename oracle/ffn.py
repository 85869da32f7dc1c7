"""Oracle: grouped expert FFN, SwiGLU and ReLU forms (test infrastructure, CPU only).

The expert FFN is the Mixtral-style SwiGLU block the paper models (Section 3.4
lists SwiGLU among the Mixtral features it models; Background: the FFN time of the
bottleneck GPU grows with the skewness).  For a row x served by expert e:
    g = x W1_e,  u = x W3_e,  h = g / (1 + exp(-g)) * u,  y = h W2_e
with no biases.  Everything is fp64 on the exact input values and nothing is
rounded in between.  The matrix products are numpy's fp64 matmul (a library
primitive used as one step); ``ffn_rows_naive`` spells the same thing as loops
and the tests tie the two together.
"""
import numpy as np


def ffn_rows(x_rows, W1_e, W3_e, W2_e):
    """y[R, d] (fp64) for rows x_rows[R, d], all served by the one expert whose
    weights are W1_e, W3_e [d, ffn] and W2_e [ffn, d]."""
    x = np.asarray(x_rows, dtype=np.float64)
    g = x @ np.asarray(W1_e, dtype=np.float64)
    u = x @ np.asarray(W3_e, dtype=np.float64)
    h = g / (1.0 + np.exp(-g)) * u
    return h @ np.asarray(W2_e, dtype=np.float64)


def ffn_rows_naive(x_rows, W1_e, W3_e, W2_e):
    """The same definition as plain Python loops (tiny inputs only)."""
    import math
    R, d = len(x_rows), len(x_rows[0])
    ffn = len(W2_e)
    y = [[0.0] * d for _ in range(R)]
    for r in range(R):
        h = [0.0] * ffn
        for f in range(ffn):
            g = 0.0
            u = 0.0
            for c in range(d):
                g += float(x_rows[r][c]) * float(W1_e[c][f])
                u += float(x_rows[r][c]) * float(W3_e[c][f])
            h[f] = g / (1.0 + math.exp(-g)) * u
        for c in range(d):
            acc = 0.0
            for f in range(ffn):
                acc += h[f] * float(W2_e[f][c])
            y[r][c] = acc
    return y


def ffn_rows_relu(x_rows, W1_e, W2_e):
    """The Switch-Transformer form of the expert FFN (Discussion, "Generality across
    model architectures": Switch Transformer uses ReLU in its FFN): y = max(x W1_e, 0) W2_e,
    no gate matrix, no biases; fp64."""
    x = np.asarray(x_rows, dtype=np.float64)
    h = np.maximum(x @ np.asarray(W1_e, dtype=np.float64), 0.0)
    return h @ np.asarray(W2_e, dtype=np.float64)


def ffn_rows_relu_naive(x_rows, W1_e, W2_e):
    """The same as plain Python loops (tiny inputs only)."""
    R, d = len(x_rows), len(x_rows[0])
    ffn = len(W2_e)
    y = [[0.0] * d for _ in range(R)]
    for r in range(R):
        h = [0.0] * ffn
        for f in range(ffn):
            g = 0.0
            for c in range(d):
                g += float(x_rows[r][c]) * float(W1_e[c][f])
            h[f] = g if g > 0.0 else 0.0
        for c in range(d):
            acc = 0.0
            for f in range(ffn):
                acc += h[f] * float(W2_e[f][c])
            y[r][c] = acc
    return y


def grouped_ffn(x_perm, seg_offsets, slot_expert, W1, W3, W2, seg_begin=0, seg_end=None):
    """y_perm[A, d] (fp64): every segment's rows go through the FFN of the expert
    that segment's slot hosts.  W1, W3: [E, d, ffn]; W2: [E, ffn, d]; W3 = None selects
    the ReLU form without a gate matrix.  Rows of segments outside [seg_begin, seg_end)
    are left at zero."""
    x_perm = np.asarray(x_perm)
    A, d = x_perm.shape
    nseg = len(slot_expert)
    if seg_end is None:
        seg_end = nseg
    y = np.zeros((A, d), dtype=np.float64)
    for s in range(seg_begin, seg_end):
        lo, hi = int(seg_offsets[s]), int(seg_offsets[s + 1])
        if hi == lo:
            continue
        e = int(slot_expert[s])
        assert e >= 0, "rows in an empty slot"
        if W3 is None:
            y[lo:hi] = ffn_rows_relu(x_perm[lo:hi], W1[e], W2[e])
        else:
            y[lo:hi] = ffn_rows(x_perm[lo:hi], W1[e], W3[e], W2[e])
    return y
