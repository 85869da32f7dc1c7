"""GPU parity of the Distribution-Only predictor (through the C ABI) against the CPU oracle:
exact integers, single calls and a stream of batches that feeds the planner."""
import numpy as np
import pytest
import torch

from oracle import route_topk, histogram, plan_duplicates, permute
from oracle.predictor import predictor_update, predictor_predict
from paper_2506_07366_amd import binding as B
from paper_2506_07366_amd import workloads as wl
from gpu_util import dev_i32

pytestmark = pytest.mark.gpu


def dev_i64(a):
    return torch.from_numpy(np.asarray(a, dtype=np.int64)).cuda()


@pytest.mark.parametrize("E,hi,A", [(1, 10, 7), (8, 1000, 8192), (64, 10**6, 49152), (128, 10**9, 262144),
                                    (1024, 10**15, 2**31 - 1), (1000, 3, 999), (5, 10**18 // 5, 2**31 - 1),
                                    (16, 100, 0), (333, 50, 1)])
def test_predict_random_counts(E, hi, A):
    rng = np.random.default_rng(E + A % 1000)
    counts = rng.integers(0, hi, size=E, endpoint=True)
    counts[rng.random(E) < 0.2] = 0
    got = B.moe_predictor_predict(dev_i64(counts), A).cpu().numpy()
    want = predictor_predict(counts.tolist(), A)
    assert got.tolist() == want
    assert int(got.sum()) == A


def test_predict_ties_and_empty_state():
    assert B.moe_predictor_predict(dev_i64([3, 3, 3]), 10).cpu().tolist() == [4, 3, 3]
    assert B.moe_predictor_predict(dev_i64([0, 0, 0, 0]), 6).cpu().tolist() == [2, 2, 1, 1]
    assert B.moe_predictor_predict(dev_i64([900, 100, 100, 100]), 8).cpu().tolist() == [6, 1, 1, 0]
    eq = [7] * 1024
    assert B.moe_predictor_predict(dev_i64(eq), 1500).cpu().tolist() == predictor_predict(eq, 1500)


def test_update_accumulates():
    rng = np.random.default_rng(2)
    E = 200
    counts = torch.zeros(E, dtype=torch.int64, device="cuda")
    ref = [0] * E
    for b in range(6):
        h = rng.integers(0, 2**31 - 1, size=E).astype(np.int32)
        B.moe_predictor_update(dev_i32(h), counts)
        ref = predictor_update(ref, h.tolist())
    assert counts.cpu().tolist() == ref


@pytest.mark.parametrize("T,E,k,G,S", [(1500, 16, 2, 4, 6), (4096, 8, 2, 8, 2), (2000, 64, 6, 8, 10)])
def test_stream_of_batches_feeds_the_planner(T, E, k, G, S):
    """predict -> plan -> permute with the predicted histogram, then learn the batch: every
    integer of every batch equals the oracle's."""
    cfg = wl.MoEConfig("stream", T=T, d=16, ffn=8, E=E, k=k, G=G, S=S, dtype="f32", mode=1, alpha=0.3, seed=21)
    counts = torch.zeros(E, dtype=torch.int64, device="cuda")
    ref_counts = [0] * E
    for b in range(5):
        logits = wl.gen_logits_batch(cfg, b)
        idx, _ = B.moe_route_topk(torch.from_numpy(logits).cuda(), k)
        hist = B.moe_histogram(idx, E)
        hp = B.moe_predictor_predict(counts, cfg.A)
        se, sq, rl, it = B.moe_plan_duplicates(1, hp, G, S, cfg.cmax)
        out = B.moe_permute(1, None, idx, None, hist, hp, se, sq, E, G, S)
        B.moe_predictor_update(hist, counts)

        ridx, _ = route_topk(logits, k)
        rhist = histogram(ridx, E)
        rhp = np.array(predictor_predict(ref_counts, cfg.A), dtype=np.int32)
        plan = plan_duplicates(1, rhp, E, G, S, cfg.cmax)
        rperm = permute(1, None, ridx, None, rhist, rhp, plan.slot_expert, plan.slot_quota, E, G, S)
        ref_counts = predictor_update(ref_counts, rhist.tolist())

        assert hp.cpu().tolist() == rhp.tolist()
        assert np.array_equal(se.cpu().numpy(), plan.slot_expert)
        assert np.array_equal(sq.cpu().numpy(), plan.slot_quota)
        assert np.array_equal(out["seg_offsets"].cpu().numpy(), rperm["seg_offsets"])
        assert np.array_equal(out["row_of_assign"].cpu().numpy(), rperm["row_of_assign"])
        assert counts.cpu().tolist() == ref_counts
