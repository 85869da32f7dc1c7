"""Pins for the grouped FFN, combine and whole-layer oracle (CPU)."""
import numpy as np
import pytest
import torch

from conftest import read_golden
from oracle import grouped_ffn, ffn_rows, combine, moe_layer, route_topk, histogram
from oracle.ffn import ffn_rows_naive
from paper_2506_07366_amd import workloads as wl


def test_ffn_rows_equals_naive_loops():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 5))
    W1 = rng.standard_normal((5, 4))
    W3 = rng.standard_normal((5, 4))
    W2 = rng.standard_normal((4, 5))
    y = ffn_rows(x, W1, W3, W2)
    yn = np.array(ffn_rows_naive(x.tolist(), W1.tolist(), W3.tolist(), W2.tolist()))
    assert np.allclose(y, yn, rtol=1e-13, atol=1e-13)
    # swapping the gate and up matrices must change the result (silu is on W1's branch)
    assert not np.allclose(y, ffn_rows(x, W3, W1, W2))


def test_ffn_closed_forms():
    # scalar case: x=2, W1=1 -> g=2, W3=3 -> u=6, W2=0.5: y = silu(2)*6*0.5
    y = ffn_rows([[2.0]], [[1.0]], [[3.0]], [[0.5]])
    assert y[0, 0] == pytest.approx(2.0 / (1.0 + np.exp(-2.0)) * 6.0 * 0.5, rel=1e-15)
    # W1 = 0 -> silu(0) = 0 -> output 0
    rng = np.random.default_rng(1)
    x = rng.standard_normal((4, 6))
    W3 = rng.standard_normal((6, 3))
    W2 = rng.standard_normal((3, 6))
    assert np.all(ffn_rows(x, np.zeros((6, 3)), W3, W2) == 0.0)
    # huge positive gate: silu(g) -> g, so y = (x W1 * x W3) W2: a plain library product
    W1 = np.abs(rng.standard_normal((6, 3))) * 1e3
    xp = np.abs(x)
    ref = ((xp @ W1) * (xp @ W3)) @ W2
    assert np.allclose(ffn_rows(xp, W1, W3, W2), ref, rtol=1e-12)


def test_single_expert_reduces_to_dense_swiglu_mlp():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((17, 12))
    W1 = rng.standard_normal((1, 12, 20)) * 0.3
    W3 = rng.standard_normal((1, 12, 20)) * 0.3
    W2 = rng.standard_normal((1, 20, 12)) * 0.3
    y = grouped_ffn(x, [0, 17], [0], W1, W3, W2)
    tx = torch.from_numpy(x)
    ref = (torch.nn.functional.silu(tx @ torch.from_numpy(W1[0])) * (tx @ torch.from_numpy(W3[0]))) \
        @ torch.from_numpy(W2[0])
    assert np.allclose(y, ref.numpy(), rtol=1e-12, atol=1e-12)


def test_grouped_uses_the_segments_expert_and_skips_empty():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((6, 4))
    W1 = rng.standard_normal((3, 4, 5))
    W3 = rng.standard_normal((3, 4, 5))
    W2 = rng.standard_normal((3, 5, 4))
    seg_offsets = [0, 2, 2, 5, 6]
    slot_expert = [2, -1, 0, 2]
    y = grouped_ffn(x, seg_offsets, slot_expert, W1, W3, W2)
    assert np.allclose(y[0:2], ffn_rows(x[0:2], W1[2], W3[2], W2[2]))
    assert np.allclose(y[2:5], ffn_rows(x[2:5], W1[0], W3[0], W2[0]))
    assert np.allclose(y[5:6], ffn_rows(x[5:6], W1[2], W3[2], W2[2]))
    # a slot range computes only its own segments
    y1 = grouped_ffn(x, seg_offsets, slot_expert, W1, W3, W2, seg_begin=2, seg_end=3)
    assert np.all(y1[0:2] == 0) and np.all(y1[5:] == 0) and np.allclose(y1[2:5], y[2:5])


def test_combine_pins():
    rng = np.random.default_rng(4)
    T, k, d = 9, 3, 5
    A = T * k
    y = rng.standard_normal((A, d))
    perm = rng.permutation(A).astype(np.int32)
    w = rng.random((T, k))
    out = combine(y, perm, w, T, k)
    for t in range(T):
        ref = sum(w[t, j] * y[perm[t * k + j]] for j in range(k))
        assert np.allclose(out[t], ref, rtol=1e-14)
    # k = 1, weight 1: a pure un-permute, exact
    p1 = rng.permutation(T).astype(np.int32)
    out1 = combine(y[:T], p1, np.ones((T, 1)), T, 1)
    assert np.array_equal(out1, y[:T][p1])


def test_identity_ffn_round_trip():
    """permute followed by combine with y_perm := x_perm returns x (weights sum to 1)."""
    from oracle import plan_duplicates, permute
    cfg = wl.MoEConfig("rt", T=64, d=8, ffn=8, E=6, k=3, G=3, S=3, dtype="f32", mode=1, seed=8)
    idx, w = route_topk(wl.gen_logits(cfg), cfg.k)
    hist = histogram(idx, cfg.E)
    plan = plan_duplicates(1, hist, cfg.E, cfg.G, cfg.S, cfg.G)
    x = wl.gen_x(cfg).astype(np.float64)
    r = permute(1, x, idx, None, hist, hist, plan.slot_expert, plan.slot_quota, cfg.E, cfg.G, cfg.S)
    out = combine(r["x_perm"], r["row_of_assign"], w, cfg.T, cfg.k)
    assert np.allclose(out, x, rtol=1e-13, atol=1e-13)


def test_layer_output_does_not_depend_on_plan_mode():
    """Replicas hold identical weights, so duplication must not change the layer's
    output; it equals the plain dense-loop definition of a top-k MoE layer."""
    cfg = wl.MoEConfig("layer", T=40, d=12, ffn=10, E=6, k=2, G=3, S=3, dtype="f32", mode=1,
                       alpha=0.3, sigma_pred=0.3, acc=0.7, seed=9)
    logits = wl.gen_logits(cfg)
    x = wl.gen_x(cfg)
    Ws = [wl.gen_expert_weights(cfg, e) for e in range(cfg.E)]
    W1 = np.stack([w[0] for w in Ws]); W3 = np.stack([w[1] for w in Ws]); W2 = np.stack([w[2] for w in Ws])
    idx, w = route_topk(logits, cfg.k)
    hist = histogram(idx, cfg.E)
    outs = []
    for mode in (0, 1, 2):
        c = cfg.replace(mode=mode)
        res = moe_layer(mode, logits, x, W1, W3, W2, cfg.k, cfg.G, cfg.S, cfg.cmax,
                        hist_pred=wl.gen_pred_hist(c, hist), pred_idx=wl.gen_pred_idx(c, idx))
        outs.append(res["out"])
    # direct definition: out[t] = sum_j w[t,j] * FFN_{idx[t,j]}(x[t])
    ref = np.zeros((cfg.T, cfg.d))
    for t in range(cfg.T):
        for j in range(cfg.k):
            e = idx[t, j]
            ref[t] += w[t, j] * ffn_rows(x[t:t + 1], W1[e], W3[e], W2[e])[0]
    for o in outs:
        assert np.allclose(o, ref, rtol=1e-12, atol=1e-14)


def test_expert_bytes_arithmetic():
    g = read_golden("expert_bytes.txt")
    assert 4096 * 14336 * 2 * 2 == g["bytes"][0]
    assert g["bytes"][0] / g["link_bytes_per_s"][0] * 1e3 == pytest.approx(g["ms"][0], rel=0.2)


# ---------------------------------------------------------------- ReLU form (Switch-Transformer FFN)
def test_relu_ffn_equals_naive_loops_and_torch():
    from oracle.ffn import ffn_rows_relu, ffn_rows_relu_naive
    rng = np.random.default_rng(20)
    x = rng.standard_normal((4, 6))
    W1 = rng.standard_normal((6, 5))
    W2 = rng.standard_normal((5, 6))
    y = ffn_rows_relu(x, W1, W2)
    yn = np.array(ffn_rows_relu_naive(x.tolist(), W1.tolist(), W2.tolist()))
    assert np.allclose(y, yn, rtol=1e-13, atol=1e-13)
    ref = torch.relu(torch.from_numpy(x) @ torch.from_numpy(W1)) @ torch.from_numpy(W2)
    assert np.allclose(y, ref.numpy(), rtol=1e-13, atol=1e-13)


def test_relu_ffn_closed_forms():
    from oracle.ffn import ffn_rows_relu
    # scalar: x=2, W1=3 -> h=6, W2=0.5 -> 3; negative pre-activation -> 0
    assert ffn_rows_relu([[2.0]], [[3.0]], [[0.5]])[0, 0] == 3.0
    assert ffn_rows_relu([[2.0]], [[-3.0]], [[0.5]])[0, 0] == 0.0
    rng = np.random.default_rng(21)
    x = np.abs(rng.standard_normal((5, 7)))
    W1 = np.abs(rng.standard_normal((7, 4)))
    W2 = rng.standard_normal((4, 7))
    # all pre-activations positive: the block is the plain product of the three matrices
    assert np.allclose(ffn_rows_relu(x, W1, W2), x @ W1 @ W2, rtol=1e-13)
    # all negative: zero
    assert np.all(ffn_rows_relu(x, -W1, W2) == 0.0)
    # positively homogeneous: f(a x) = a f(x) for a > 0 (not true of the SwiGLU form)
    assert np.allclose(ffn_rows_relu(3.0 * x, W1 - 0.5, W2), 3.0 * ffn_rows_relu(x, W1 - 0.5, W2), rtol=1e-12)


def test_grouped_relu_uses_the_segments_expert():
    from oracle.ffn import ffn_rows_relu
    rng = np.random.default_rng(22)
    x = rng.standard_normal((6, 4))
    W1 = rng.standard_normal((3, 4, 5))
    W2 = rng.standard_normal((3, 5, 4))
    y = grouped_ffn(x, [0, 2, 2, 6], [2, -1, 0], W1, None, W2)
    assert np.array_equal(y[0:2], ffn_rows_relu(x[0:2], W1[2], W2[2]))
    assert np.array_equal(y[2:6], ffn_rows_relu(x[2:6], W1[0], W2[0]))
