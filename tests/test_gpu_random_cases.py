"""Seeded random cases of every stage against the oracle (shapes, segment sizes around the tile
edges, empty slots, slot ranges, both FFN forms, the fused gather and gate weights, all three
plan modes, rank counts on both sides of the planner's two versions)."""
import numpy as np
import pytest
import torch

from paper_2506_07366_amd import binding as B, workloads as wl
from paper_2506_07366_amd.layer import to_device
from oracle import grouped_ffn, histogram, permute, plan_duplicates, route_topk
from oracle.comm import comm_matrices
from oracle.predictor import predictor_predict

pytestmark = pytest.mark.gpu


def _i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_ffn_cases(seed):
    rng = np.random.default_rng(seed)
    for it in range(40):
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        d = int(rng.choice([64, 128, 192, 256, 512])) if dtype == "bf16" else int(rng.choice([4, 36, 64, 128]))
        ffn = int(rng.choice([8, 20, 64, 96, 128, 200, 256, 320, 688, 1100])) if dtype == "bf16" else int(rng.choice([4, 20, 64, 132]))
        E = int(rng.integers(1, 9))
        nseg = int(rng.integers(1, 40))
        sizes = rng.choice([0, 0, 1, 2, 31, 32, 33, 64, 100, 127, 128, 129, 200, 255, 256, 257, 300, 513, 700], size=nseg)
        if sizes.sum() == 0:
            sizes[0] = 5
        slot_expert = [int(rng.integers(0, E)) if s > 0 or rng.random() < 0.5 else -1 for s in sizes]
        relu = bool(rng.random() < 0.4)
        A = int(sizes.sum())
        so = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
        x = wl.quantize(rng.standard_normal((A, d)).astype(np.float32), dtype)
        W1 = wl.quantize((rng.standard_normal((E, d, ffn)) * 0.1).astype(np.float32), dtype)
        W3 = wl.quantize((rng.standard_normal((E, d, ffn)) * 0.1).astype(np.float32), dtype)
        W2 = wl.quantize((rng.standard_normal((E, ffn, d)) * 0.1).astype(np.float32), dtype)
        dev = lambda a: to_device(wl.to_storage(a, dtype), dtype)
        packed = B.moe_pack_weights_relu(dev(W1), dev(W2)) if relu else B.moe_pack_weights(dev(W1), dev(W3), dev(W2))
        b0, b1 = 0, nseg
        if rng.random() < 0.3:
            b0 = int(rng.integers(0, nseg))
            b1 = int(rng.integers(b0, nseg + 1))
        # any tile shape for either product, the second product whole, by the rule or split everywhere
        B.moe_grouped_ffn_set_option(B.FFN_OPT_TILE1, int(rng.integers(-1, 3)))
        B.moe_grouped_ffn_set_option(B.FFN_OPT_TILE2, int(rng.integers(-1, 3)))
        B.moe_grouped_ffn_set_option(B.FFN_OPT_SPLIT_K, int(rng.integers(-1, 2)))
        try:
            ref = grouped_ffn(x, so, slot_expert, W1, None if relu else W3, W2, b0, b1)
            y = B.moe_grouped_ffn(dev(x), _i32(so), _i32(slot_expert), packed, E, ffn, b0, b1, relu=relu)
            tol = 2e-2 if dtype == "bf16" else 1e-5
            lo, hi = int(so[b0]), int(so[b1])
            what = dict(seed=seed, it=it, dtype=dtype, d=d, ffn=ffn, E=E, sizes=sizes.tolist(), relu=relu, b0=b0, b1=b1)
            if hi > lo:
                err = np.max(np.abs(y.float().cpu().numpy()[lo:hi] - ref[lo:hi])) / max(np.max(np.abs(ref)), 1e-30)
                assert err <= tol, what
            if not relu and dtype == "bf16":
                # rows gathered through a random assignment map, with and without gate weights
                k = int(rng.integers(1, 4))
                T = -(-A // k)
                a_of_row = np.zeros(T * k, dtype=np.int32)
                a_of_row[:] = rng.permutation(T * k)
                x_src = wl.quantize(rng.standard_normal((T, d)).astype(np.float32), dtype)
                xg = x_src[a_of_row[:A] // k]
                ref2 = grouped_ffn(xg, so, slot_expert, W1, W3, W2)
                if T * k == A:
                    y2 = B.moe_grouped_ffn_gather(dev(x_src), _i32(a_of_row), k, _i32(so), _i32(slot_expert), packed, E, ffn)
                    err2 = np.max(np.abs(y2.float().cpu().numpy()[:A] - ref2)) / max(np.max(np.abs(ref2)), 1e-30)
                    assert err2 <= tol, what
                    wts = rng.random((T, k)).astype(np.float32)
                    y3 = B.moe_grouped_ffn_gather(dev(x_src), _i32(a_of_row), k, _i32(so), _i32(slot_expert), packed, E, ffn,
                                                  topk_w=torch.from_numpy(wts).cuda())
                    ref3 = ref2 * wts.reshape(-1)[a_of_row[:A]][:, None]
                    err3 = np.max(np.abs(y3.float().cpu().numpy()[:A] - ref3)) / max(np.max(np.abs(ref3)), 1e-30)
                    assert err3 <= tol, what
        finally:
            for opt in (B.FFN_OPT_TILE1, B.FFN_OPT_TILE2, B.FFN_OPT_SPLIT_K):
                B.moe_grouped_ffn_set_option(opt, -1)


@pytest.mark.parametrize("seed", [21, 22])
def test_random_integer_stage_cases(seed):
    rng = np.random.default_rng(seed)
    done = 0
    while done < 120:
        E = int(rng.choice([1, 2, 3, 5, 8, 16, 33, 64, 100, 128, 257, 512, 1024]))
        G = int(rng.choice([1, 2, 3, 4, 7, 8, 16, 32, 64, 65, 100, 256]))
        H = -(-E // G)
        if H > 16:
            continue
        S = int(rng.integers(H, min(16, H + 4) + 1))
        if G * S > 2048:
            continue
        k = int(rng.integers(1, min(E, 16) + 1))
        T = int(rng.choice([1, 2, 63, 64, 65, 300, 1000, 2047, 2049, 5000, 20000]))
        if T * k > 60000:
            T = max(1, 60000 // k)
        mode = int(rng.integers(0, 3))
        cmax = int(rng.integers(1, G + 1))
        cfg = wl.MoEConfig("random", T=T, d=16, ffn=8, E=E, k=k, G=G, S=S, dtype="f32", mode=mode,
                           alpha=float(rng.choice([0.05, 0.3, 1.0, 10.0])), sigma_pred=float(rng.choice([0.0, 0.2, 1.0])),
                           acc=float(rng.choice([0.0, 0.5, 0.9, 1.0])), seed=int(rng.integers(0, 10**6)), c_max=cmax)
        what = dict(seed=seed, case=done, T=T, E=E, k=k, G=G, S=S, mode=mode, cmax=cmax, cfg_seed=cfg.seed)
        logits = wl.gen_logits(cfg)
        if done % 5 == 0:
            logits = (np.round(logits * 2) / 2).astype(np.float32)  # many ties
        ridx, rw = route_topk(logits, k)
        rhist = histogram(ridx, E)
        pi = wl.gen_pred_idx(cfg, ridx) if mode == 2 else None
        if mode == 2:
            rhp = histogram(pi, E)
        elif mode == 1:
            rhp = wl.gen_pred_hist(cfg, rhist) if done % 3 else np.array(predictor_predict(rhist.tolist(), cfg.A), dtype=np.int32)
        else:
            rhp = rhist
        plan = plan_duplicates(mode, rhp, E, G, S, cfg.cmax)
        rp = permute(mode, None, ridx, pi, rhist, rhp, plan.slot_expert, plan.slot_quota, E, G, S)
        rd, rc = comm_matrices(mode, ridx, pi, rp["row_of_assign"], rp["seg_offsets"], G, S)
        idx, w = B.moe_route_topk(torch.from_numpy(logits).cuda(), k)
        hist = B.moe_histogram(idx, E)
        dpi = None if pi is None else _i32(pi)
        hp = B.moe_histogram(dpi, E) if mode == 2 else _i32(rhp)
        se, sq, rl, ni = B.moe_plan_duplicates(mode, hp, G, S, cfg.cmax)
        out = B.moe_permute(mode, None, idx, dpi, hist, hp, se, sq, E, G, S)
        dd, dc = B.moe_comm_matrix(mode, idx, dpi, out["row_of_assign"], out["seg_offsets"], G, S)
        assert np.array_equal(idx.cpu().numpy(), ridx), what
        assert float(np.max(np.abs(w.cpu().numpy() - rw))) <= 1e-6, what
        assert np.array_equal(hist.cpu().numpy(), rhist), what
        assert np.array_equal(se.cpu().numpy(), plan.slot_expert) and np.array_equal(sq.cpu().numpy(), plan.slot_quota), what
        assert int(ni.item()) == plan.n_iters, what
        assert np.array_equal(out["seg_offsets"].cpu().numpy(), rp["seg_offsets"]), what
        assert np.array_equal(out["row_of_assign"].cpu().numpy(), rp["row_of_assign"]), what
        assert np.array_equal(out["assign_of_row"].cpu().numpy(), rp["assign_of_row"]), what
        assert np.array_equal(dd.cpu().numpy(), rd) and np.array_equal(dc.cpu().numpy(), rc), what
        done += 1
