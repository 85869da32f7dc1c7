"""GPU parity, stage by stage: the HIP path through the C ABI against the CPU oracle
on the same seeded inputs.  Integer results must match bit for bit."""
import numpy as np
import pytest
import torch

from oracle import route_topk, histogram, plan_duplicates, permute, combine, home_slot
from oracle.comm import comm_matrices
from paper_2506_07366_amd import binding as B
from paper_2506_07366_amd import workloads as wl
from gpu_util import Case, dev_i32, to_host_f32

pytestmark = pytest.mark.gpu

ALL_CFGS = list(wl.CONFIGS)
INT_CFGS = ["cfg1_tiny_f32", "cfg2_mixtral_dist", "cfg3_mixtral_t2e", "cfg4_finegrained", "mid_bf16"] + \
    [n for n in wl.CONFIGS if n.startswith("cfg5")]


# ---------------------------------------------------------------- routing
@pytest.mark.parametrize("E,k,T", [(8, 2, 1000), (64, 6, 777), (128, 8, 513), (5, 5, 100), (7, 1, 64), (1, 1, 10),
                                   (2, 2, 33), (16, 4, 129), (33, 3, 65), (200, 16, 70), (1024, 8, 40),
                                   (300, 5, 1), (48, 3, 100), (34, 2, 50), (96, 6, 333), (256, 8, 100),
                                   (512, 16, 30), (513, 7, 20), (17, 16, 70), (128, 16, 4099)])
def test_route_random(E, k, T):
    rng = np.random.default_rng(E * 1000 + k)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    idx, w = B.moe_route_topk(torch.from_numpy(logits).cuda(), k)
    ridx, rw = route_topk(logits, k)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    assert np.max(np.abs(w.cpu().numpy().astype(np.float64) - rw)) <= 1e-6


def test_route_ties_lowest_index():
    rng = np.random.default_rng(1)
    for E, k in [(16, 4), (128, 8), (8, 2), (64, 6), (40, 5), (512, 16), (1000, 9)]:
        logits = (np.round(rng.standard_normal((500, E)) * 2) / 4).astype(np.float32)
        logits[0, :] = 0.0                      # an all-equal row
        idx, w = B.moe_route_topk(torch.from_numpy(logits).cuda(), k)
        ridx, rw = route_topk(logits, k)
        assert np.array_equal(idx.cpu().numpy(), ridx)
        assert list(idx[0].cpu().numpy()) == list(range(k))
        assert np.max(np.abs(w.cpu().numpy() - rw)) <= 1e-6


def test_route_signed_zeros_denormals_and_k_equal_E():
    """Values that compare equal without being the same bits (+0 and -0), values below the normal
    range, very large magnitudes and k = E (every logit is taken once, none twice)."""
    rng = np.random.default_rng(7)
    for E, k in [(8, 8), (16, 16), (24, 16), (128, 8), (64, 6), (5, 3), (32, 16), (3, 3)]:
        logits = rng.standard_normal((300, E)).astype(np.float32)
        zero_mask = rng.random((300, E)) < 0.4
        logits[zero_mask] = np.where(rng.random(int(zero_mask.sum())) < 0.5, np.float32(0.0), np.float32(-0.0))
        tiny = rng.random((300, E)) < 0.2
        logits[tiny] = (rng.integers(-6, 7, int(tiny.sum())) * np.float32(1e-41)).astype(np.float32)  # subnormal steps
        logits[1, :] = np.float32(-0.0)
        logits[2, :] = np.float32(-3.0e38)
        logits[3, : E // 2] = np.float32(3.0e38)
        idx, w = B.moe_route_topk(torch.from_numpy(logits).cuda(), k)
        ridx, rw = route_topk(logits, k)
        got = idx.cpu().numpy()
        assert np.array_equal(got, ridx), (E, k)
        assert all(len(set(r)) == k for r in got)
        assert np.max(np.abs(w.cpu().numpy().astype(np.float64) - rw)) <= 1e-6


@pytest.mark.parametrize("name", INT_CFGS)
def test_integer_stages_on_config(name):
    """route, histogram, plan and permutation on the full-size seeded workload."""
    cfg = wl.CONFIGS[name]
    case = Case(cfg, with_x=False)
    idx, w = B.moe_route_topk(case.dev_logits(), cfg.k)
    assert np.array_equal(idx.cpu().numpy(), case.idx)
    assert np.max(np.abs(w.cpu().numpy().astype(np.float64) - case.w)) <= 1e-6
    hist = B.moe_histogram(idx, cfg.E)
    assert np.array_equal(hist.cpu().numpy(), case.hist)
    assert int(hist.sum()) == cfg.A

    pred_idx = case.dev_pred_idx()
    if cfg.mode == wl.MODE_TOKEN:
        hp = B.moe_histogram(pred_idx, cfg.E)
        assert np.array_equal(hp.cpu().numpy(), case.hist_plan)
    else:
        hp = case.dev_hist_plan()
    se, sq, rl, it = B.moe_plan_duplicates(cfg.mode, hp, cfg.G, cfg.S, cfg.cmax)
    assert np.array_equal(se.cpu().numpy(), case.plan.slot_expert)
    assert np.array_equal(sq.cpu().numpy(), case.plan.slot_quota)
    assert np.array_equal(rl.cpu().numpy(), case.plan.rank_load_pred)
    assert int(it.item()) == case.plan.n_iters

    out = B.moe_permute(cfg.mode, None, idx, pred_idx, hist, hp, se, sq, cfg.E, cfg.G, cfg.S)
    assert np.array_equal(out["seg_offsets"].cpu().numpy(), case.perm["seg_offsets"])
    assert np.array_equal(out["row_of_assign"].cpu().numpy(), case.perm["row_of_assign"])
    assert np.array_equal(out["assign_of_row"].cpu().numpy(), case.perm["assign_of_row"])
    assert np.array_equal(out["rank_load"].cpu().numpy(), case.perm["rank_load"])
    assert int(out["rank_load"].sum()) == cfg.A

    # rows crossing the emulated ranks, from the permutation just computed
    disp, comb = B.moe_comm_matrix(cfg.mode, idx, pred_idx if cfg.mode == wl.MODE_TOKEN else None,
                                   out["row_of_assign"], out["seg_offsets"], cfg.G, cfg.S)
    rdisp, rcomb = comm_matrices(cfg.mode, case.idx, case.pred_idx, case.perm["row_of_assign"],
                                 case.perm["seg_offsets"], cfg.G, cfg.S)
    assert np.array_equal(disp.cpu().numpy(), rdisp)
    assert np.array_equal(comb.cpu().numpy(), rcomb)
    assert np.array_equal(disp.cpu().numpy().sum(axis=0), case.perm["rank_load"])


# ---------------------------------------------------------------- histogram
@pytest.mark.parametrize("n,E", [(0, 4), (1, 1), (100, 8), (65536, 64), (65537, 64), (300001, 128), (70000, 1024)])
def test_histogram_sizes(n, E):
    rng = np.random.default_rng(n + E)
    idx = rng.integers(0, E, size=n).astype(np.int32)
    h = B.moe_histogram(torch.from_numpy(idx).cuda(), E)
    assert np.array_equal(h.cpu().numpy(), histogram(idx, E))
    # not accumulated across calls
    h2 = B.moe_histogram(torch.from_numpy(idx).cuda(), E, out=h)
    assert np.array_equal(h2.cpu().numpy(), histogram(idx, E))


# ---------------------------------------------------------------- plan
def test_plan_random_small_cases():
    rng = np.random.default_rng(17)
    for trial in range(60):
        E = int(rng.integers(1, 40))
        G = int(rng.integers(1, 20))
        H = -(-E // G)
        S = H + int(rng.integers(0, 4))
        if S > 16:
            continue
        c_max = int(rng.integers(1, G + 1))
        n = (rng.dirichlet(np.full(E, 0.3)) * rng.integers(1, 50000)).astype(np.int32)
        if trial % 7 == 0:
            n[:] = 0
        for mode in (0, 1):
            ref = plan_duplicates(mode, n, E, G, S, c_max)
            se, sq, rl, it = B.moe_plan_duplicates(mode, dev_i32(n), G, S, c_max)
            assert np.array_equal(se.cpu().numpy(), ref.slot_expert), (E, G, S, c_max, n)
            assert np.array_equal(sq.cpu().numpy(), ref.slot_quota)
            assert np.array_equal(rl.cpu().numpy(), ref.rank_load_pred)
            assert int(it.item()) == ref.n_iters


def test_plan_many_ranks():
    # more ranks than one wavefront has lanes
    rng = np.random.default_rng(3)
    E, G, S = 300, 150, 4
    n = (rng.dirichlet(np.full(E, 0.2)) * 400000).astype(np.int32)
    ref = plan_duplicates(1, n, E, G, S, G)
    se, sq, rl, it = B.moe_plan_duplicates(1, dev_i32(n), G, S, G)
    assert np.array_equal(se.cpu().numpy(), ref.slot_expert)
    assert np.array_equal(sq.cpu().numpy(), ref.slot_quota)
    assert int(it.item()) == ref.n_iters


# ---------------------------------------------------------------- permute
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("T,E,k,G,S", [(300, 12, 3, 4, 5), (1, 4, 2, 2, 2), (2049, 8, 1, 8, 2), (5000, 40, 7, 10, 6),
                                       (700, 6, 6, 3, 3), (1000, 128, 16, 32, 5),
                                       (900, 1024, 16, 256, 8),      # the limits: 1024 experts, top-16, 2048 segments
                                       (3000, 1000, 4, 128, 16),     # 16 slots per rank
                                       # whole numbers of 2048-assignment chunks and one over; 256 / 257 experts
                                       (4096, 8, 2, 8, 2), (8192, 8, 1, 8, 2), (8193, 8, 1, 8, 2),
                                       (512, 256, 16, 64, 4), (512, 257, 16, 64, 5), (2731, 64, 3, 16, 5),
                                       # both sides of the one-workgroup path's limits: 8192 assignments,
                                       # 512 experts, 512 segments
                                       (400, 512, 8, 64, 8), (400, 513, 8, 64, 9), (1024, 300, 8, 32, 16),
                                       (1024, 300, 8, 33, 16), (1, 1, 1, 1, 1), (8192, 512, 1, 128, 4),
                                       # hundreds of chunks; many chunks at the largest expert and segment counts
                                       (70000, 16, 8, 4, 5), (20000, 1024, 16, 256, 8)])
def test_permute_small(mode, T, E, k, G, S):
    cfg = wl.MoEConfig("p", T=T, d=16, ffn=8, E=E, k=k, G=G, S=S, dtype="f32", mode=mode, alpha=0.3,
                       sigma_pred=0.3, acc=0.8, seed=T + E)
    case = Case(cfg)
    x = case.dev_x()
    idx = dev_i32(case.idx)
    out = B.moe_permute(mode, x, idx, case.dev_pred_idx(), dev_i32(case.hist), case.dev_hist_plan(),
                        dev_i32(case.plan.slot_expert), dev_i32(case.plan.slot_quota), E, G, S)
    assert np.array_equal(out["seg_offsets"].cpu().numpy(), case.perm["seg_offsets"])
    assert np.array_equal(out["row_of_assign"].cpu().numpy(), case.perm["row_of_assign"])
    assert np.array_equal(out["assign_of_row"].cpu().numpy(), case.perm["assign_of_row"])
    assert np.array_equal(out["rank_load"].cpu().numpy(), case.perm["rank_load"])
    ref_rows = case.x[case.perm["assign_of_row"] // k]
    assert np.array_equal(out["x_perm"].cpu().numpy(), ref_rows)        # byte-exact row copy


def test_permute_empty_input():
    E, G, S, k = 4, 2, 2, 2
    plan = plan_duplicates(0, [0] * E, E, G, S, G)
    out = B.moe_permute(0, torch.zeros((0, 8), device="cuda"), torch.zeros((0, k), dtype=torch.int32, device="cuda"),
                        None, dev_i32([0] * E), dev_i32([0] * E), dev_i32(plan.slot_expert),
                        dev_i32(plan.slot_quota), E, G, S)
    assert out["seg_offsets"].cpu().tolist() == [0] * (G * S + 1)
    assert out["rank_load"].cpu().tolist() == [0, 0]


def test_permute_bf16_rows_byte_exact():
    cfg = wl.MoEConfig("pb", T=513, d=2048, ffn=64, E=8, k=2, G=4, S=3, dtype="bf16", mode=1, sigma_pred=0.2, seed=4)
    case = Case(cfg)
    x = case.dev_x()
    out = B.moe_permute(1, x, dev_i32(case.idx), None, dev_i32(case.hist), case.dev_hist_plan(),
                        dev_i32(case.plan.slot_expert), dev_i32(case.plan.slot_quota), cfg.E, cfg.G, cfg.S)
    got = out["x_perm"].view(torch.int16).cpu().numpy()
    ref = x.view(torch.int16).cpu().numpy()[case.perm["assign_of_row"] // cfg.k]
    assert np.array_equal(got, ref)


# ---------------------------------------------------------------- combine
@pytest.mark.parametrize("dtype,T,k,d", [("f32", 100, 3, 64), ("bf16", 257, 2, 4096), ("bf16", 50, 8, 136),
                                         ("f32", 7, 1, 4), ("bf16", 31, 16, 512)])
def test_combine(dtype, T, k, d):
    rng = np.random.default_rng(T + k + d)
    A = T * k
    y = wl.quantize(rng.standard_normal((A, d)).astype(np.float32), dtype)
    rows = rng.permutation(A).astype(np.int32)
    w = rng.random((T, k)).astype(np.float32)
    w /= w.sum(axis=1, keepdims=True)
    from paper_2506_07366_amd.layer import to_device
    out = B.moe_combine(to_device(wl.to_storage(y, dtype), dtype), dev_i32(rows), torch.from_numpy(w).cuda(), T, k)
    ref = combine(y, rows, w, T, k)
    tol = 1e-5 if dtype == "f32" else 2e-2
    assert np.max(np.abs(to_host_f32(out) - ref)) <= tol * np.max(np.abs(ref))
    if k == 1:
        # weight-one un-permute is byte exact
        out1 = B.moe_combine(to_device(wl.to_storage(y, dtype), dtype), dev_i32(rows),
                             torch.ones((T, 1), device="cuda"), T, 1)
        assert np.array_equal(to_host_f32(out1), y[rows])


# ---------------------------------------------------------------- cross-rank traffic
@pytest.mark.parametrize("mode,T,E,k,G,S", [(0, 1, 1, 1, 1, 1), (1, 333, 12, 3, 4, 5), (2, 333, 12, 3, 4, 5),
                                            (2, 5000, 64, 6, 8, 10), (1, 2000, 256, 4, 128, 4),
                                            (2, 1500, 256, 8, 256, 2), (0, 777, 10, 2, 5, 2)])
def test_comm_matrix_small(mode, T, E, k, G, S):
    cfg = wl.MoEConfig("comm", T=T, d=16, ffn=8, E=E, k=k, G=G, S=S, dtype="f32", mode=mode, alpha=0.3,
                       sigma_pred=0.3, acc=0.7, seed=11)
    case = Case(cfg, with_x=False)
    idx = dev_i32(case.idx)
    pred_idx = case.dev_pred_idx()
    disp, comb = B.moe_comm_matrix(mode, idx, pred_idx if mode == wl.MODE_TOKEN else None,
                                   dev_i32(case.perm["row_of_assign"]), dev_i32(case.perm["seg_offsets"]), G, S)
    rdisp, rcomb = comm_matrices(mode, case.idx, case.pred_idx, case.perm["row_of_assign"],
                                 case.perm["seg_offsets"], G, S)
    assert np.array_equal(disp.cpu().numpy(), rdisp)
    assert np.array_equal(comb.cpu().numpy(), rcomb)


def test_comm_matrix_empty_batch():
    z = torch.zeros((0, 2), dtype=torch.int32, device="cuda")
    so = torch.zeros(4 * 2 + 1, dtype=torch.int32, device="cuda")
    disp, comb = B.moe_comm_matrix(0, z, None, torch.zeros(0, dtype=torch.int32, device="cuda"), so, 4, 2)
    assert int(disp.abs().sum()) == 0 and int(comb.abs().sum()) == 0


# ---------------------------------------------------------------- pessimistic prediction errors
def test_errors_concentrated_on_one_rank():
    """Section 3.3, pessimistic case: every mispredicted assignment belongs to an expert homed
    on rank 0, so all the fall-back rows pile up there.  Integers equal the oracle's, and the
    bottleneck is worse than with the same number of errors spread at random."""
    cfg = wl.MoEConfig("pess", T=6000, d=16, ffn=8, E=64, k=6, G=8, S=10, dtype="f32", mode=2, alpha=1.0,
                       acc=0.85, seed=13)
    on_rank0 = np.array([home_slot(e, cfg.E, cfg.G, cfg.S) // cfg.S == 0 for e in range(cfg.E)])
    worst = Case(cfg, with_x=False, pred_idx=lambda idx: wl.gen_pred_idx_concentrated(cfg, idx, on_rank0))
    typical = Case(cfg, with_x=False)
    n_wrong = int((worst.pred_idx != worst.idx).sum())
    assert n_wrong > 0

    idx = dev_i32(worst.idx)
    pred = dev_i32(worst.pred_idx)
    hist = B.moe_histogram(idx, cfg.E)
    hp = B.moe_histogram(pred, cfg.E)
    se, sq, rl, it = B.moe_plan_duplicates(2, hp, cfg.G, cfg.S, cfg.cmax)
    out = B.moe_permute(2, None, idx, pred, hist, hp, se, sq, cfg.E, cfg.G, cfg.S)
    assert np.array_equal(se.cpu().numpy(), worst.plan.slot_expert)
    assert np.array_equal(out["row_of_assign"].cpu().numpy(), worst.perm["row_of_assign"])
    assert np.array_equal(out["rank_load"].cpu().numpy(), worst.perm["rank_load"])
    disp, comb = B.moe_comm_matrix(2, idx, pred, out["row_of_assign"], out["seg_offsets"], cfg.G, cfg.S)
    rdisp, rcomb = comm_matrices(2, worst.idx, worst.pred_idx, worst.perm["row_of_assign"],
                                 worst.perm["seg_offsets"], cfg.G, cfg.S)
    assert np.array_equal(disp.cpu().numpy(), rdisp) and np.array_equal(comb.cpu().numpy(), rcomb)
    # every transfer at dispatch ends on rank 0
    off = rdisp - np.diag(np.diag(rdisp))
    assert off[:, 1:].sum() == 0 and off[:, 0].sum() > 0
    load = worst.perm["rank_load"]
    assert load.argmax() == 0
    assert load.max() > typical.perm["rank_load"].max()


# ---------------------------------------------------------------- determinism
def test_integer_stages_do_not_depend_on_the_launch():
    """Every integer output is byte-identical from run to run and between batches cut in different
    ways: no position is decided by an atomic or by arrival order.  The first 3000 tokens of a
    5000-token batch routed alone give the first 3000 rows of its routing (another grid), the
    histogram of a concatenation is the sum of the parts' (wide and single-workgroup kernels), and
    plan and permutation repeat bit for bit."""
    cfg = wl.MoEConfig("det", T=5000, d=64, ffn=64, E=40, k=7, G=10, S=6, dtype="f32", mode=2, alpha=0.3, acc=0.8,
                       seed=77)
    case = Case(cfg)
    lg = case.dev_logits()
    idx1, w1 = B.moe_route_topk(lg, cfg.k)
    idx2, w2 = B.moe_route_topk(lg, cfg.k)
    assert torch.equal(idx1, idx2) and torch.equal(w1.view(torch.int32), w2.view(torch.int32))
    idx3, w3 = B.moe_route_topk(lg[:3000].contiguous(), cfg.k)
    assert torch.equal(idx3, idx1[:3000]) and torch.equal(w3.view(torch.int32), w1[:3000].view(torch.int32))
    big = idx1.repeat(12, 1)                                        # 420 000 ids: the wide histogram kernel
    h_big = B.moe_histogram(big, cfg.E)
    h_one = B.moe_histogram(idx1, cfg.E)                            # 35 000 ids: one workgroup
    assert torch.equal(h_big, 12 * h_one) and torch.equal(h_one, B.moe_histogram(idx1, cfg.E))
    pred = case.dev_pred_idx()
    hp = B.moe_histogram(pred, cfg.E)
    plans = [B.moe_plan_duplicates(2, hp, cfg.G, cfg.S, cfg.cmax) for _ in range(2)]
    for a, b in zip(*plans):
        assert torch.equal(a, b)
    se, sq = plans[0][0], plans[0][1]
    outs = [B.moe_permute(2, case.dev_x(), idx1, pred, h_one, hp, se, sq, cfg.E, cfg.G, cfg.S) for _ in range(2)]
    for key in ("seg_offsets", "row_of_assign", "assign_of_row", "rank_load", "x_perm"):
        assert torch.equal(outs[0][key].view(torch.uint8), outs[1][key].view(torch.uint8)), key
