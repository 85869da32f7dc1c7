"""GPU parity of the grouped SwiGLU FFN and of the whole layer against the fp64 oracle.

Tolerances: max|delta| <= 1e-5 * max|ref| for fp32 and <= 2e-2 * max|ref| for bf16
storage with fp32 accumulation (hidden activation and output rounded to bf16)."""
import numpy as np
import pytest
import torch

from oracle import grouped_ffn, ffn_rows, combine, moe_layer
from oracle.histogram import skewness
from oracle.ffn import ffn_rows_relu
from paper_2506_07366_amd import binding as B
from paper_2506_07366_amd import workloads as wl
from paper_2506_07366_amd.layer import MoELayer, to_device
from gpu_util import Case, dev_i32, to_host_f32, weights_storage, shape_key

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


@pytest.fixture
def ffn_options():
    """Sets overrides of the grouped FFN's automatic choices and restores the defaults afterwards."""
    def set_(tile1=-1, tile2=-1, split=-1, group_n=0):
        B.moe_grouped_ffn_set_option(B.FFN_OPT_TILE1, tile1)
        B.moe_grouped_ffn_set_option(B.FFN_OPT_TILE2, tile2)
        B.moe_grouped_ffn_set_option(B.FFN_OPT_SPLIT_K, split)
        B.moe_grouped_ffn_set_option(B.FFN_OPT_GROUP_N, group_n)
    yield set_
    set_()


def expert_row_lists(seg_offsets, slot_expert, E):
    """Rows of x_perm per expert in the order the FFN tiles them: segments of the expert in
    ascending slot id, rows ascending."""
    lists = [[] for _ in range(E)]
    for s_, e in enumerate(slot_expert):
        if 0 <= e < E:
            lists[e].extend(range(int(seg_offsets[s_]), int(seg_offsets[s_ + 1])))
    return lists


def host_weights(cfg):
    W1s, W3s, W2s = weights_storage(shape_key(cfg))
    return W1s, W3s, W2s


def dev_weights(cfg, Ws):
    return tuple(to_device(w, cfg.dtype) for w in Ws)


def rel_err(got, ref):
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))


def run_ffn_case(cfg, seg_sizes, slot_expert, seed=0):
    """x_perm with the given ragged segments through the HIP FFN and the oracle."""
    rng = np.random.default_rng(seed)
    A = int(sum(seg_sizes))
    x = wl.quantize(rng.standard_normal((A, cfg.d)).astype(np.float32), cfg.dtype)
    seg_offsets = np.concatenate([[0], np.cumsum(seg_sizes)]).astype(np.int32)
    Ws = host_weights(cfg)
    packed = B.moe_pack_weights(*dev_weights(cfg, Ws))
    y = B.moe_grouped_ffn(to_device(wl.to_storage(x, cfg.dtype), cfg.dtype), dev_i32(seg_offsets),
                          dev_i32(slot_expert), packed, cfg.E, cfg.ffn)
    Wf = [wl.from_storage(w, cfg.dtype) for w in Ws]
    ref = grouped_ffn(x, seg_offsets, slot_expert, *Wf)
    return to_host_f32(y), ref, seg_offsets


@pytest.mark.parametrize("dtype,d,ffn", [("f32", 128, 256), ("f32", 36, 20), ("bf16", 128, 256), ("bf16", 512, 1024),
                                         ("bf16", 64, 64), ("bf16", 192, 1408), ("bf16", 128, 688), ("bf16", 64, 20),
                                         ("bf16", 256, 1376)])
def test_ffn_ragged_segments(dtype, d, ffn):
    E = 5
    cfg = wl.MoEConfig("f", T=1, d=d, ffn=ffn, E=E, k=1, G=4, S=3, dtype=dtype, mode=0, seed=21)
    # sizes around the tile edges (64/128/256) and empty segments; an empty slot (-1) with no rows
    seg_sizes = [1, 0, 127, 129, 0, 256, 257, 63, 300, 0, 5, 64]
    slot_expert = [0, 1, 2, 3, -1, 4, 0, 1, 2, 3, 4, 0]
    got, ref, so = run_ffn_case(cfg, seg_sizes, slot_expert)
    assert rel_err(got, ref) <= TOL[dtype]
    # per-row check too (a wrong expert or a dropped tail row must not hide behind the global max)
    scale = np.max(np.abs(ref))
    assert np.all(np.max(np.abs(got - ref), axis=1) <= TOL[dtype] * scale)


def test_ffn_slot_range_only_touches_its_rows():
    cfg = wl.MoEConfig("f", T=1, d=128, ffn=256, E=5, k=1, G=4, S=3, dtype="bf16", mode=0, seed=21)
    rng = np.random.default_rng(5)
    seg_sizes = [40, 0, 130, 7, 0, 200, 33, 0, 64, 1, 0, 90]
    slot_expert = [0, -1, 2, 3, -1, 4, 0, -1, 2, 3, -1, 1]
    A = sum(seg_sizes)
    x = wl.quantize(rng.standard_normal((A, cfg.d)).astype(np.float32), "bf16")
    so = np.concatenate([[0], np.cumsum(seg_sizes)]).astype(np.int32)
    Ws = host_weights(cfg)
    packed = B.moe_pack_weights(*dev_weights(cfg, Ws))
    xd = to_device(wl.to_storage(x, "bf16"), "bf16")
    y_full = B.moe_grouped_ffn(xd, dev_i32(so), dev_i32(slot_expert), packed, cfg.E, cfg.ffn)
    y_rank = B.moe_grouped_ffn(xd, dev_i32(so), dev_i32(slot_expert), packed, cfg.E, cfg.ffn, seg_begin=3, seg_end=6)
    yf, yr = to_host_f32(y_full), to_host_f32(y_rank)
    assert np.array_equal(yr[so[3]:so[6]], yf[so[3]:so[6]])
    assert np.all(yr[:so[3]] == 0) and np.all(yr[so[6]:] == 0)


@pytest.mark.parametrize("name", ["cfg1_tiny_f32", "mid_bf16"])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_layer_full_compare(name, mode):
    """Whole path on configs the oracle finishes in full."""
    cfg = wl.CONFIGS[name].replace(mode=mode, acc=0.9, sigma_pred=wl.CONFIGS[name].sigma_pred)
    case = Case(cfg)
    Ws = host_weights(cfg)
    Wf = [wl.from_storage(w, cfg.dtype) for w in Ws]
    ref = moe_layer(mode, case.logits, case.x, *Wf, cfg.k, cfg.G, cfg.S, cfg.cmax,
                    hist_pred=case.hist_plan, pred_idx=case.pred_idx)
    layer = MoELayer(cfg)
    layer.set_weights(*dev_weights(cfg, Ws))
    out = layer.step(case.dev_logits(), case.dev_x(), hist_pred=case.dev_hist_plan(), pred_idx=case.dev_pred_idx())
    torch.cuda.synchronize()
    assert np.array_equal(layer.topk_idx.cpu().numpy(), ref["topk_idx"])
    assert np.array_equal(layer.perm["row_of_assign"].cpu().numpy(), ref["perm"]["row_of_assign"])
    assert np.array_equal(layer.slot_expert.cpu().numpy(), ref["plan"].slot_expert)
    assert rel_err(to_host_f32(layer.y_perm), ref["y_perm"]) <= TOL[cfg.dtype]
    assert rel_err(to_host_f32(out), ref["out"]) <= TOL[cfg.dtype]
    rep = layer.load_report()
    assert rep["makespan"] == int(ref["perm"]["rank_load"].max())
    assert rep["n_iters"] == ref["plan"].n_iters
    assert rep["skewness"] == pytest.approx(skewness(ref["hist"] if "hist" in ref else case.hist), rel=1e-12)
    assert rep["imbalance"] == pytest.approx(float(ref["perm"]["rank_load"].max()) * cfg.G / cfg.A, rel=1e-12)


FULL = ["cfg2_mixtral_dist", "cfg3_mixtral_t2e", "cfg4_finegrained"] + \
       [f"cfg5_prefill_a{a}_m{m}" for a in ("0.1", "1", "10") for m in (0, 1, 2)] + \
       ["cfg5_decode_m0", "cfg5_decode_m1", "cfg5_decode_m2", "cfg6_switch_relu", "cfg7_llama_moe"]


@pytest.mark.parametrize("name", FULL)
def test_layer_full_size_sampled(name):
    """Full-size configs in the launch configuration the benchmark times: integer
    outputs compared in full, FFN / layer outputs on sampled rows the oracle can
    compute one by one: all k rows of sampled tokens, the first and last row of
    every non-empty segment, and the rows either side of every tile boundary the
    kernels can use (rows are tiled per expert, over all its segments, in tiles of
    256 or 128 rows: every multiple of 128 in every expert's row list).  The load
    report is compared with the oracle's skewness and rank loads."""
    cfg = wl.CONFIGS[name]
    case = Case(cfg)
    Ws = host_weights(cfg)
    layer = MoELayer(cfg)
    layer.set_weights(*dev_weights(cfg, Ws))
    out = layer.step(case.dev_logits(), case.dev_x(), hist_pred=case.dev_hist_plan(), pred_idx=case.dev_pred_idx())
    torch.cuda.synchronize()
    assert np.array_equal(layer.topk_idx.cpu().numpy(), case.idx)
    assert np.array_equal(layer.hist.cpu().numpy(), case.hist)
    assert np.array_equal(layer.slot_expert.cpu().numpy(), case.plan.slot_expert)
    assert np.array_equal(layer.slot_quota.cpu().numpy(), case.plan.slot_quota)
    assert np.array_equal(layer.perm["seg_offsets"].cpu().numpy(), case.perm["seg_offsets"])
    assert np.array_equal(layer.perm["row_of_assign"].cpu().numpy(), case.perm["row_of_assign"])
    assert np.array_equal(layer.perm["rank_load"].cpu().numpy(), case.perm["rank_load"])

    rng = np.random.default_rng(123)
    n_tok = min(cfg.T, 128)
    toks = np.sort(rng.choice(cfg.T, size=n_tok, replace=False))
    roa = case.perm["row_of_assign"].reshape(cfg.T, cfg.k)
    rows = set(roa[toks].reshape(-1).tolist())
    so = case.perm["seg_offsets"]
    for s in range(cfg.nseg):
        lo, hi = int(so[s]), int(so[s + 1])
        if hi > lo:
            rows.update([lo, hi - 1])
    for lst in expert_row_lists(so, case.plan.slot_expert, cfg.E):
        for b in range(128, len(lst), 128):       # every tile boundary inside the expert's rows
            rows.update([lst[b - 1], lst[b]])
    rows = np.array(sorted(rows), dtype=np.int64)
    aor = case.perm["assign_of_row"]
    seg_of_row = np.searchsorted(so, rows, side="right") - 1
    exp_of_row = case.plan.slot_expert[seg_of_row]
    assert np.array_equal(exp_of_row, case.idx.reshape(-1)[aor[rows]])
    y_ref = np.zeros((rows.size, cfg.d))
    for e in np.unique(exp_of_row):
        sel = np.nonzero(exp_of_row == e)[0]
        xr = case.x[aor[rows[sel]] // cfg.k]
        if cfg.act == "relu":
            y_ref[sel] = ffn_rows_relu(xr, wl.from_storage(Ws[0][e], cfg.dtype), wl.from_storage(Ws[2][e], cfg.dtype))
        else:
            y_ref[sel] = ffn_rows(xr, wl.from_storage(Ws[0][e], cfg.dtype), wl.from_storage(Ws[1][e], cfg.dtype),
                                  wl.from_storage(Ws[2][e], cfg.dtype))
    y_got = to_host_f32(layer.y_perm[torch.from_numpy(rows).cuda()])
    scale = np.max(np.abs(y_ref))
    assert np.all(np.max(np.abs(y_got - y_ref), axis=1) <= TOL[cfg.dtype] * scale)
    # layer output of the sampled tokens
    pos = {int(r): i for i, r in enumerate(rows)}
    out_ref = np.zeros((n_tok, cfg.d))
    for i, t in enumerate(toks):
        for j in range(cfg.k):
            out_ref[i] += case.w[t, j] * y_ref[pos[int(roa[t, j])]]
    out_got = to_host_f32(out[torch.from_numpy(toks).cuda()])
    assert np.max(np.abs(out_got - out_ref)) <= TOL[cfg.dtype] * np.max(np.abs(out_ref))
    # properties that hold at any size
    assert int(layer.perm["rank_load"].sum()) == cfg.A
    assert torch.isfinite(out.float()).all()
    # load report against the oracle: skewness of the histogram, bottleneck rank over the mean
    rep = layer.load_report()
    assert rep["skewness"] == pytest.approx(skewness(case.hist), rel=1e-12)
    assert rep["imbalance"] == pytest.approx(float(case.perm["rank_load"].max()) * cfg.G / cfg.A, rel=1e-12)
    assert rep["makespan"] == int(case.perm["rank_load"].max())
    assert rep["rank_load"] == case.perm["rank_load"].tolist()


def test_output_independent_of_plan_mode():
    """Replicas hold the same weights: the layer output must not depend on the plan."""
    cfg = wl.CONFIGS["mid_bf16"]
    Ws = host_weights(cfg)
    outs = []
    for mode in (0, 1, 2):
        c = cfg.replace(mode=mode, acc=0.8)
        case = Case(c)
        layer = MoELayer(c)
        layer.set_weights(*dev_weights(c, Ws))
        out = layer.step(case.dev_logits(), case.dev_x(), hist_pred=case.dev_hist_plan(),
                         pred_idx=case.dev_pred_idx())
        outs.append(to_host_f32(out))
    scale = np.max(np.abs(outs[0]))
    assert np.max(np.abs(outs[1] - outs[0])) <= 2e-2 * scale
    assert np.max(np.abs(outs[2] - outs[0])) <= 2e-2 * scale


def test_identity_round_trip_permute_combine():
    """permute then combine with y_perm := x_perm returns x (gate weights sum to 1)."""
    cfg = wl.MoEConfig("rt", T=777, d=256, ffn=64, E=16, k=4, G=4, S=6, dtype="f32", mode=1, sigma_pred=0.3, seed=6)
    case = Case(cfg)
    x = case.dev_x()
    idx, w = B.moe_route_topk(case.dev_logits(), cfg.k)
    out = B.moe_permute(1, x, idx, None, dev_i32(case.hist), case.dev_hist_plan(), dev_i32(case.plan.slot_expert),
                        dev_i32(case.plan.slot_quota), cfg.E, cfg.G, cfg.S)
    back = B.moe_combine(out["x_perm"], out["row_of_assign"], w, cfg.T, cfg.k)
    assert np.max(np.abs(to_host_f32(back) - case.x)) <= 1e-5 * np.max(np.abs(case.x))


@pytest.mark.parametrize("name,mode", [("cfg1_tiny_f32", 1), ("mid_bf16", 0), ("mid_bf16", 1), ("mid_bf16", 2),
                                       ("cfg4_finegrained", 1)])
def test_fused_gather_equals_copied_rows(name, mode):
    """Gathering the token rows inside the first product must give exactly what the
    FFN gives on the copied rows (same arithmetic on the same values)."""
    cfg = wl.CONFIGS[name].replace(mode=mode, acc=0.9)
    case = Case(cfg)
    Ws = host_weights(cfg)
    dw = dev_weights(cfg, Ws)
    outs = []
    for fused in (False, True):
        layer = MoELayer(cfg, fused_gather=fused)
        layer.set_weights(*dw)
        out = layer.step(case.dev_logits(), case.dev_x(), hist_pred=case.dev_hist_plan(),
                         pred_idx=case.dev_pred_idx())
        torch.cuda.synchronize()
        outs.append((layer.y_perm.float().cpu().numpy().copy(), out.float().cpu().numpy().copy()))
        assert np.array_equal(layer.perm["row_of_assign"].cpu().numpy(), case.perm["row_of_assign"])
    assert np.array_equal(outs[0][0], outs[1][0])
    assert np.array_equal(outs[0][1], outs[1][1])


def test_fused_gather_slot_range_and_oracle():
    cfg = wl.CONFIGS["mid_bf16"]
    case = Case(cfg)
    Ws = host_weights(cfg)
    Wf = [wl.from_storage(w, cfg.dtype) for w in Ws]
    layer = MoELayer(cfg, fused_gather=True)
    layer.set_weights(*dev_weights(cfg, Ws))
    layer.step(case.dev_logits(), case.dev_x(), hist_pred=case.dev_hist_plan(), pred_idx=None)
    x_perm = case.x[case.perm["assign_of_row"] // cfg.k]
    ref = grouped_ffn(x_perm, case.perm["seg_offsets"], case.plan.slot_expert, *Wf)
    assert rel_err(to_host_f32(layer.y_perm), ref) <= TOL["bf16"]
    # one rank's slots alone
    layer.y_perm.zero_()
    layer.ffn(seg_begin=cfg.S, seg_end=2 * cfg.S)
    so = case.perm["seg_offsets"]
    got = to_host_f32(layer.y_perm)
    lo, hi = so[cfg.S], so[2 * cfg.S]
    assert rel_err(got[lo:hi], ref[lo:hi]) <= TOL["bf16"]
    assert np.all(got[:lo] == 0) and np.all(got[hi:] == 0)


# ---------------------------------------------------------------- ReLU form of the FFN
@pytest.mark.parametrize("dtype,d,ffn", [("f32", 128, 256), ("f32", 36, 20), ("bf16", 128, 256), ("bf16", 512, 1024),
                                         ("bf16", 64, 64), ("bf16", 768, 3072), ("bf16", 192, 1408), ("bf16", 128, 688),
                                         ("bf16", 64, 8)])
def test_relu_ffn_ragged_segments(dtype, d, ffn):
    E = 5
    cfg = wl.MoEConfig("f", T=1, d=d, ffn=ffn, E=E, k=1, G=4, S=3, dtype=dtype, mode=0, seed=21, act="relu")
    seg_sizes = [1, 0, 127, 129, 0, 256, 257, 63, 300, 0, 5, 64]
    slot_expert = [0, 1, 2, 3, -1, 4, 0, 1, 2, 3, 4, 0]
    rng = np.random.default_rng(3)
    A = int(sum(seg_sizes))
    x = wl.quantize(rng.standard_normal((A, d)).astype(np.float32), dtype)
    seg_offsets = np.concatenate([[0], np.cumsum(seg_sizes)]).astype(np.int32)
    W1s, _, W2s = host_weights(cfg)
    packed = B.moe_pack_weights_relu(to_device(W1s, dtype), to_device(W2s, dtype))
    y = B.moe_grouped_ffn(to_device(wl.to_storage(x, dtype), dtype), dev_i32(seg_offsets), dev_i32(slot_expert),
                          packed, E, ffn, relu=True)
    ref = grouped_ffn(x, seg_offsets, slot_expert, wl.from_storage(W1s, dtype), None, wl.from_storage(W2s, dtype))
    got = to_host_f32(y)
    scale = np.max(np.abs(ref))
    assert np.all(np.max(np.abs(got - ref), axis=1) <= TOL[dtype] * scale)
    # the SwiGLU entry point on the same rows gives something else: the two forms are not mixed up
    assert scale > 0


def test_relu_layer_top1_full_compare():
    """A small top-1 ReLU layer end to end against the oracle (every output element)."""
    cfg = wl.MoEConfig("switch_small", T=700, d=128, ffn=256, E=12, k=1, G=4, S=4, dtype="bf16", mode=1, alpha=0.3,
                       sigma_pred=0.2, seed=31, act="relu")
    case = Case(cfg)
    Ws = host_weights(cfg)
    layer = MoELayer(cfg)
    layer.set_weights(*dev_weights(cfg, Ws))
    out = layer.step(case.dev_logits(), case.dev_x(), hist_pred=case.dev_hist_plan(), pred_idx=None)
    ref = moe_layer(cfg.mode, case.logits, case.x, wl.from_storage(Ws[0], cfg.dtype), None,
                    wl.from_storage(Ws[2], cfg.dtype), cfg.k, cfg.G, cfg.S, cfg.cmax, hist_pred=case.hist_plan)
    assert np.array_equal(layer.perm["row_of_assign"].cpu().numpy(), ref["perm"]["row_of_assign"])
    assert rel_err(to_host_f32(layer.y_perm), ref["y_perm"]) <= TOL[cfg.dtype]
    assert rel_err(to_host_f32(out), ref["out"]) <= TOL[cfg.dtype]
    # top-1: the gate weight is exactly 1, the layer output is the expert output of the token's row
    assert np.all(case.w == 1.0)


def test_ffn_many_tiny_segments():
    """2048 segments (the limit) of 0..5 rows each: every M-tile is a ragged one."""
    rng = np.random.default_rng(8)
    E, d, ffn, nseg = 32, 64, 64, 2048
    cfg = wl.MoEConfig("tiny", T=1, d=d, ffn=ffn, E=E, k=1, G=256, S=8, dtype="bf16", mode=0, seed=23)
    seg_sizes = rng.integers(0, 6, size=nseg).tolist()
    slot_expert = [int(e) if n > 0 or rng.random() < 0.5 else -1 for e, n in zip(rng.integers(0, E, size=nseg), seg_sizes)]
    got, ref, so = run_ffn_case(cfg, seg_sizes, slot_expert, seed=9)
    scale = np.max(np.abs(ref))
    assert np.all(np.max(np.abs(got - ref), axis=1) <= TOL["bf16"] * scale)


@pytest.mark.parametrize("split", [-1, 1])
def test_ffn_many_experts_full_and_ragged_tiles(split, ffn_options):
    """1024 experts (the limit) over 2048 segments, a few experts with several full-height tiles and
    several segments, the rest slivers: every expert's ragged tile has to find its place among a
    thousand others, with and without tiles split along K."""
    ffn_options(split=split)
    rng = np.random.default_rng(18)
    E, d, ffn, nseg = 1024, 64, 256, 2048
    cfg = wl.MoEConfig("many", T=1, d=d, ffn=ffn, E=E, k=1, G=256, S=8, dtype="bf16", mode=0, seed=24)
    seg_sizes = rng.integers(0, 4, size=nseg)
    slot_expert = rng.integers(0, E, size=nseg)
    big = rng.choice(nseg, size=12, replace=False)
    seg_sizes[big] = rng.integers(200, 700, size=12)
    slot_expert[big] = rng.integers(0, 5, size=12)          # several segments of the same few experts
    slot_expert = [int(e) if n > 0 or rng.random() < 0.5 else -1 for e, n in zip(slot_expert, seg_sizes)]
    got, ref, so = run_ffn_case(cfg, [int(n) for n in seg_sizes], slot_expert, seed=19)
    scale = np.max(np.abs(ref))
    assert np.all(np.max(np.abs(got - ref), axis=1) <= TOL["bf16"] * scale)


def test_ffn_one_huge_segment_and_empty_rest():
    """All rows in the last of 12 segments: 20 full-height tiles of one expert, nothing else."""
    cfg = wl.MoEConfig("huge", T=1, d=128, ffn=256, E=5, k=1, G=4, S=3, dtype="bf16", mode=0, seed=21)
    seg_sizes = [0] * 11 + [5120]
    slot_expert = [0, 1, 2, 3, -1, 4, 0, 1, 2, 3, 4, 2]
    got, ref, so = run_ffn_case(cfg, seg_sizes, slot_expert, seed=10)
    scale = np.max(np.abs(ref))
    assert np.all(np.max(np.abs(got - ref), axis=1) <= TOL["bf16"] * scale)


@pytest.mark.parametrize("split", [0, 1])
@pytest.mark.parametrize("tile2", [0, 1, 2])
@pytest.mark.parametrize("tile1", [0, 1, 2])
def test_ffn_every_tile_variant(tile1, tile2, split, ffn_options):
    """The tile shapes built into the library (forced through moe_grouped_ffn_set_option) all
    compute the same FFN, with the closing tiles of the second product computed whole (0) or as
    parts of K added up afterwards (1: forced; 320 hidden columns are 5 k-tiles, so the four
    parts are unequal)."""
    ffn_options(tile1=tile1, tile2=tile2, split=split)
    cfg = wl.MoEConfig("v", T=1, d=256, ffn=320, E=5, k=1, G=4, S=3, dtype="bf16", mode=0, seed=21)
    seg_sizes = [1, 0, 127, 129, 0, 256, 257, 63, 300, 0, 5, 64]
    slot_expert = [0, 1, 2, 3, -1, 4, 0, 1, 2, 3, 4, 0]
    got, ref, so = run_ffn_case(cfg, seg_sizes, slot_expert, seed=tile1 * 3 + tile2)
    scale = np.max(np.abs(ref))
    assert np.all(np.max(np.abs(got - ref), axis=1) <= TOL["bf16"] * scale)


@pytest.mark.parametrize("relu", [False, True])
def test_ffn_split_k_matches_whole_tiles(relu, ffn_options):
    """Closing tiles computed as parts of K: same result as whole tiles up to the fp32
    association of the partial sums (one bf16 rounding step of the output), rows outside the
    slot range untouched, and the same answer on a second run (the order in which workgroups
    claim tiles does not reach the result)."""
    cfg = wl.MoEConfig("s", T=1, d=192, ffn=688, E=4, k=1, G=4, S=3, dtype="bf16", mode=0, seed=29)
    rng = np.random.default_rng(31)
    seg_sizes = [300, 0, 256, 1, 513, 0, 77, 255, 128, 0, 31, 640]
    slot_expert = [0, -1, 2, 3, 1, 2, 0, 1, 2, -1, 3, 0]
    A = sum(seg_sizes)
    x = wl.quantize(rng.standard_normal((A, cfg.d)).astype(np.float32), "bf16")
    so = np.concatenate([[0], np.cumsum(seg_sizes)]).astype(np.int32)
    W1s, W3s, W2s = host_weights(cfg)
    if relu:
        packed = B.moe_pack_weights_relu(to_device(W1s, "bf16"), to_device(W2s, "bf16"))
    else:
        packed = B.moe_pack_weights(*dev_weights(cfg, (W1s, W3s, W2s)))
    xd = to_device(wl.to_storage(x, "bf16"), "bf16")
    out = {}
    for split in (0, 1):
        ffn_options(split=split)
        out[split] = to_host_f32(B.moe_grouped_ffn(xd, dev_i32(so), dev_i32(slot_expert), packed, cfg.E, cfg.ffn,
                                                   relu=relu))
        again = to_host_f32(B.moe_grouped_ffn(xd, dev_i32(so), dev_i32(slot_expert), packed, cfg.E, cfg.ffn,
                                              relu=relu))
        assert np.array_equal(out[split], again)
        out[split, "range"] = to_host_f32(B.moe_grouped_ffn(xd, dev_i32(so), dev_i32(slot_expert), packed, cfg.E,
                                                            cfg.ffn, seg_begin=3, seg_end=8, relu=relu))
    Wf = [wl.from_storage(w, "bf16") for w in (W1s, W3s, W2s)]
    ref = grouped_ffn(x, so, slot_expert, Wf[0], None if relu else Wf[1], Wf[2])
    scale = np.max(np.abs(ref))
    for split in (0, 1):
        assert np.all(np.max(np.abs(out[split] - ref), axis=1) <= TOL["bf16"] * scale)
        r = out[split, "range"]
        assert np.max(np.abs(r[so[3]:so[8]] - ref[so[3]:so[8]])) <= TOL["bf16"] * scale
        assert np.all(r[:so[3]] == 0) and np.all(r[so[8]:] == 0)
    # whole (unsplit) tiles accumulate a row's products in the same order whatever else is launched
    # with them: the slot range alone gives the same bits as the full launch
    assert np.array_equal(out[0, "range"][so[3]:so[8]], out[0][so[3]:so[8]])
    assert np.max(np.abs(out[0] - out[1])) <= 2.0 ** -7 * scale


def test_ffn_replicas_of_one_expert_share_tiles():
    """Several segments of the range host the same expert (replicas hold the same weights):
    their rows are tiled together, whatever their sizes, and every row still gets its own
    expert's result; a row's result does not depend on which replica served it."""
    cfg = wl.MoEConfig("r", T=1, d=128, ffn=256, E=4, k=1, G=6, S=2, dtype="bf16", mode=0, seed=37)
    seg_sizes = [3, 200, 0, 58, 130, 1, 256, 7, 0, 90, 511, 2]
    slot_expert = [0, 1, 0, 0, 2, 0, 1, 0, -1, 3, 0, 1]      # expert 0 in seven slots, one of them empty
    got, ref, so = run_ffn_case(cfg, seg_sizes, slot_expert, seed=12)
    scale = np.max(np.abs(ref))
    assert np.all(np.max(np.abs(got - ref), axis=1) <= TOL["bf16"] * scale)
    # the same rows with every segment on its own (one launch per slot): same values up to the
    # position of the rows inside their tiles, which does not change a row's sum
    rng = np.random.default_rng(12)
    x = wl.quantize(rng.standard_normal((int(sum(seg_sizes)), cfg.d)).astype(np.float32), "bf16")
    Ws = host_weights(cfg)
    packed = B.moe_pack_weights(*dev_weights(cfg, Ws))
    xd = to_device(wl.to_storage(x, "bf16"), "bf16")
    y = torch.zeros_like(xd)
    for s_ in range(len(seg_sizes)):
        B.moe_grouped_ffn(xd, dev_i32(so), dev_i32(slot_expert), packed, cfg.E, cfg.ffn, seg_begin=s_, seg_end=s_ + 1,
                          out=y)
    assert np.array_equal(to_host_f32(y), got)


@pytest.mark.parametrize("name,mode", [("cfg1_tiny_f32", 1), ("mid_bf16", 0), ("mid_bf16", 1), ("mid_bf16", 2)])
def test_fused_gate_weights_against_oracle(name, mode):
    """Gate weights applied by the second product (moe_grouped_ffn_fused) and a plain sum in
    moe_combine: the layer output against the oracle's combine of the oracle's FFN, and the
    weighted rows against w * (oracle row).  Rule for the bits: fp32 rows are exactly
    fl(w * y) of the unweighted path's y; bf16 rows are rounded once from w * (fp32 sum), so
    they differ from bf16(w * bf16(y)) by at most one rounding step."""
    cfg = wl.CONFIGS[name].replace(mode=mode, acc=0.9)
    case = Case(cfg)
    Ws = host_weights(cfg)
    Wf = [wl.from_storage(w, cfg.dtype) for w in Ws]
    ref = moe_layer(mode, case.logits, case.x, *Wf, cfg.k, cfg.G, cfg.S, cfg.cmax,
                    hist_pred=case.hist_plan, pred_idx=case.pred_idx)
    dw = dev_weights(cfg, Ws)
    plain = MoELayer(cfg, fused_gather=True)
    plain.set_weights(*dw)
    plain.step(case.dev_logits(), case.dev_x(), hist_pred=case.dev_hist_plan(), pred_idx=case.dev_pred_idx())
    fused = MoELayer(cfg, fused_weights=True)
    fused.set_weights(*dw)
    out = fused.step(case.dev_logits(), case.dev_x(), hist_pred=case.dev_hist_plan(), pred_idx=case.dev_pred_idx())
    torch.cuda.synchronize()
    assert rel_err(to_host_f32(out), ref["out"]) <= TOL[cfg.dtype]
    w_row = case.w.reshape(-1)[ref["perm"]["assign_of_row"]]                 # gate weight of every row
    yw_ref = ref["y_perm"] * w_row[:, None]
    yw = to_host_f32(fused.y_perm)
    assert np.max(np.abs(yw - yw_ref)) <= TOL[cfg.dtype] * np.max(np.abs(ref["y_perm"]))
    y_plain = to_host_f32(plain.y_perm)
    w32 = fused.topk_w.cpu().numpy().reshape(-1)[ref["perm"]["assign_of_row"]].astype(np.float32)
    if cfg.dtype == "f32":
        assert np.array_equal(yw, y_plain * w32[:, None])
    else:
        twice = wl.quantize(y_plain * w32[:, None], "bf16")                  # rounded twice: bf16(w * bf16(sum))
        step = np.maximum(np.abs(yw), np.abs(twice)) * 2.0 ** -7             # a bf16 rounding step at that size
        assert np.all(np.abs(yw - twice) <= 2 * step + 1e-30)


def test_fused_gate_weights_full_size_sampled():
    """The fused path (row gather in the first product, gate weights in the second, plain sum
    in the combine) at the headline size: layer output of sampled tokens against the oracle."""
    cfg = wl.CONFIGS["cfg2_mixtral_dist"]
    case = Case(cfg)
    Ws = host_weights(cfg)
    layer = MoELayer(cfg, fused_weights=True)
    layer.set_weights(*dev_weights(cfg, Ws))
    out = layer.step(case.dev_logits(), case.dev_x(), hist_pred=case.dev_hist_plan(), pred_idx=case.dev_pred_idx())
    torch.cuda.synchronize()
    assert np.array_equal(layer.perm["row_of_assign"].cpu().numpy(), case.perm["row_of_assign"])
    rng = np.random.default_rng(77)
    toks = np.sort(rng.choice(cfg.T, size=96, replace=False))
    out_ref = np.zeros((toks.size, cfg.d))
    for i, t in enumerate(toks):
        for j in range(cfg.k):
            e = int(case.idx[t, j])
            y = ffn_rows(case.x[t:t + 1], wl.from_storage(Ws[0][e], cfg.dtype), wl.from_storage(Ws[1][e], cfg.dtype),
                         wl.from_storage(Ws[2][e], cfg.dtype))
            out_ref[i] += case.w[t, j] * y[0]
    out_got = to_host_f32(out[torch.from_numpy(toks).cuda()])
    assert np.max(np.abs(out_got - out_ref)) <= TOL["bf16"] * np.max(np.abs(out_ref))


@pytest.mark.parametrize("split", [-1, 1])
def test_ffn_workspace_exact_size_accepted_one_byte_less_refused(split, ffn_options):
    """The size moe_grouped_ffn_workspace_bytes reports is what the call needs: a caller-owned
    workspace of exactly that size works, one byte less is refused before anything is launched."""
    ffn_options(split=split)
    cfg = wl.MoEConfig("w", T=1, d=128, ffn=256, E=3, k=1, G=2, S=2, dtype="bf16", mode=0, seed=33)
    rng = np.random.default_rng(34)
    seg_sizes = [70, 300, 0, 129]
    slot_expert = [0, 1, -1, 2]
    A = sum(seg_sizes)
    x = wl.quantize(rng.standard_normal((A, cfg.d)).astype(np.float32), "bf16")
    so = np.concatenate([[0], np.cumsum(seg_sizes)]).astype(np.int32)
    Ws = host_weights(cfg)
    packed = B.moe_pack_weights(*dev_weights(cfg, Ws))
    xd = to_device(wl.to_storage(x, "bf16"), "bf16")
    need = B.moe_grouped_ffn_workspace_bytes(A, cfg.d, cfg.ffn, len(seg_sizes), 1)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    y = to_host_f32(B.moe_grouped_ffn(xd, dev_i32(so), dev_i32(slot_expert), packed, cfg.E, cfg.ffn, workspace=ws))
    Wf = [wl.from_storage(w, "bf16") for w in Ws]
    ref = grouped_ffn(x, so, slot_expert, *Wf)
    assert np.all(np.max(np.abs(y - ref), axis=1) <= TOL["bf16"] * np.max(np.abs(ref)))
    with pytest.raises(B.MoeGpsError):
        B.moe_grouped_ffn(xd, dev_i32(so), dev_i32(slot_expert), packed, cfg.E, cfg.ffn, workspace=ws[:need - 1])


def test_ffn_bits_do_not_depend_on_the_order_tiles_are_claimed():
    """Workgroups claim tiles from counters, so the order varies from run to run; a row's sums
    do not: ten runs of a Mixtral-shaped batch give the same bytes, split tiles included."""
    cfg = wl.CONFIGS["cfg2_mixtral_dist"].replace(T=1024)
    case = Case(cfg)
    Ws = host_weights(cfg)
    layer = MoELayer(cfg)
    layer.set_weights(*dev_weights(cfg, Ws))
    first = None
    for _ in range(10):
        out = layer.step(case.dev_logits(), case.dev_x(), hist_pred=case.dev_hist_plan(), pred_idx=case.dev_pred_idx())
        torch.cuda.synchronize()
        got = (layer.y_perm.view(torch.int16).clone(), out.view(torch.int16).clone())
        if first is None:
            first = got
        assert torch.equal(got[0], first[0]) and torch.equal(got[1], first[1])


@pytest.mark.parametrize("name,mode", [("mid_bf16", 1), ("mid_bf16", 2), ("cfg1_tiny_f32", 1)])
def test_layer_step_replays_from_a_hip_graph(name, mode):
    """The whole step captured into a HIP graph: every replay gives the eager step's bytes, also
    after the inputs were overwritten in place and with eager work and synchronisations between
    the replays."""
    cfg = wl.CONFIGS[name].replace(mode=mode, acc=0.9)
    case = Case(cfg)
    Ws = host_weights(cfg)
    dw = dev_weights(cfg, Ws)
    logits, x = case.dev_logits(), case.dev_x()
    hp, pi = case.dev_hist_plan(), case.dev_pred_idx()
    eager = MoELayer(cfg)
    eager.set_weights(*dw)
    layer = MoELayer(cfg)
    layer.set_weights(*dw)
    graph = layer.capture(logits, x, hist_pred=hp, pred_idx=pi)
    rng = np.random.default_rng(5)
    for rep in range(4):
        if rep > 0:   # new token rows and router logits in the captured tensors
            x.copy_(to_device(wl.to_storage(wl.quantize(rng.standard_normal((cfg.T, cfg.d)).astype(np.float32), cfg.dtype),
                                            cfg.dtype), cfg.dtype))
            logits.copy_(torch.from_numpy(rng.standard_normal((cfg.T, cfg.E)).astype(np.float32)).cuda())
        layer.out.zero_()
        layer.y_perm.zero_()
        torch.cuda.synchronize()
        graph.replay()
        ref = eager.step(logits, x, hist_pred=hp, pred_idx=pi)
        torch.cuda.synchronize()
        assert torch.equal(layer.topk_idx, eager.topk_idx)
        assert torch.equal(layer.perm["row_of_assign"], eager.perm["row_of_assign"])
        assert torch.equal(layer.out.view(torch.uint8), ref.view(torch.uint8)), rep
