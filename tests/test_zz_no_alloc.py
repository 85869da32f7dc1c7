"""moe_permute_static (the entry point that allocates nothing; its scratch is a fixed device
array of the library) against moe_permute on the same inputs: every output bit for bit, on
two calls in a row, the second with a smaller input, then a third in another plan mode."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2506_07366_amd import binding as B
from paper_2506_07366_amd import workloads as wl

pytestmark = pytest.mark.gpu

KEYS = ("seg_offsets", "row_of_assign", "assign_of_row", "x_perm", "rank_load")


def _inputs(cfg):
    logits = torch.from_numpy(wl.gen_logits(cfg)).cuda()
    idx, _ = B.moe_route_topk(logits, cfg.k)
    hist = B.moe_histogram(idx, cfg.E)
    x = torch.from_numpy(wl.gen_x(cfg).astype(np.float32)).cuda()
    if cfg.dtype == "bf16":
        x = x.to(torch.bfloat16)
    pred = None
    hp = hist
    if cfg.mode == wl.MODE_TOKEN:
        pred = torch.from_numpy(wl.gen_pred_idx(cfg, idx.cpu().numpy())).cuda()
        hp = B.moe_histogram(pred, cfg.E)
    elif cfg.mode == wl.MODE_DISTRIBUTION:
        hp = torch.from_numpy(wl.gen_pred_hist(cfg, hist.cpu().numpy())).cuda()
    se, sq, _, _ = B.moe_plan_duplicates(cfg.mode, hp, cfg.G, cfg.S, cfg.cmax)
    return x, idx, pred, hist, hp, se, sq


def _both(cfg):
    x, idx, pred, hist, hp, se, sq = _inputs(cfg)
    ref = B.moe_permute(cfg.mode, x, idx, pred, hist, hp, se, sq, cfg.E, cfg.G, cfg.S)
    got = B.moe_permute(cfg.mode, x, idx, pred, hist, hp, se, sq, cfg.E, cfg.G, cfg.S, static_scratch=True)
    torch.cuda.synchronize()
    for key in KEYS:
        a, b = ref[key], got[key]
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"{cfg.name}: {key} differs"
    assert int(got["seg_offsets"][-1].item()) == cfg.A


def test_static_scratch_matches_workspace_path():
    big = wl.MoEConfig("static_big", T=6000, d=256, ffn=64, E=64, k=6, G=16, S=5, dtype="bf16",
                       mode=wl.MODE_DISTRIBUTION, seed=11, sigma_pred=0.2)
    small = wl.MoEConfig("static_small", T=301, d=128, ffn=64, E=8, k=2, G=4, S=3, dtype="f32",
                         mode=wl.MODE_DISTRIBUTION, seed=12, sigma_pred=0.2)
    token = wl.MoEConfig("static_token", T=1500, d=128, ffn=64, E=16, k=4, G=8, S=3, dtype="bf16",
                         mode=wl.MODE_TOKEN, seed=13, acc=0.8)
    _both(big)      # first call on this device: looks up the array's address
    _both(small)    # smaller input right behind it: stale counters of the first call must not matter
    _both(token)
    _both(big)


def test_static_scratch_refuses_sizes_beyond_the_array():
    lib = B.load_library()
    T, E, k, G, S = 1 << 20, 128, 8, 32, 5
    assert lib.moe_permute_workspace_bytes(T, E, k, G, S) > (8 << 20)
    one = torch.zeros(1, dtype=torch.int32, device="cuda")
    p = ctypes.c_void_p(one.data_ptr())
    rc = lib.moe_permute_static(0, None, 1, T, 128, E, k, G, S, p, None, None, None, p, p, p, p, p, None, p, None)
    assert rc == -3
    torch.cuda.synchronize()
