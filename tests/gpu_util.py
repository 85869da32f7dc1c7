"""Helpers shared by the GPU parity tests: build a seeded case on the host, run the
oracle's integer stages, and move the inputs to the device."""
import functools

import numpy as np
import torch

from oracle import route_topk, histogram, plan_duplicates, permute
from paper_2506_07366_amd import workloads as wl
from paper_2506_07366_amd.layer import to_device


def have_gpu():
    return torch.cuda.is_available()


@functools.lru_cache(maxsize=2)
def weights_storage(shape_key):
    """Storage-form weights for a (seed, E, d, ffn, dtype) shape; cached because the
    sweep configs share one set of weights."""
    seed, E, d, ffn, dtype = shape_key
    cfg = wl.MoEConfig("w", T=1, d=d, ffn=ffn, E=E, k=1, G=1, S=E, dtype=dtype, mode=0, seed=seed)
    return wl.gen_weights_storage(cfg, threads=16)


def shape_key(cfg):
    return (cfg.seed, cfg.E, cfg.d, cfg.ffn, cfg.dtype)


class Case:
    """Host inputs + oracle results of the integer stages for one config."""

    def __init__(self, cfg, with_x=True, pred_idx=None):
        """``pred_idx``: a function of the true ids that replaces the config's own prediction."""
        self.cfg = cfg
        self.logits = wl.gen_logits(cfg)
        self.idx, self.w = route_topk(self.logits, cfg.k)
        self.hist = histogram(self.idx, cfg.E)
        self.pred_idx = None
        if cfg.mode == wl.MODE_TOKEN:
            self.pred_idx = wl.gen_pred_idx(cfg, self.idx) if pred_idx is None else pred_idx(self.idx)
            self.hist_plan = histogram(self.pred_idx, cfg.E)
        elif cfg.mode == wl.MODE_DISTRIBUTION:
            self.hist_plan = wl.gen_pred_hist(cfg, self.hist)
        else:
            self.hist_plan = self.hist
        self.plan = plan_duplicates(cfg.mode, self.hist_plan, cfg.E, cfg.G, cfg.S, cfg.cmax)
        self.x = wl.gen_x(cfg) if with_x else None
        self.perm = permute(cfg.mode, None, self.idx, self.pred_idx, self.hist, self.hist_plan,
                            self.plan.slot_expert, self.plan.slot_quota, cfg.E, cfg.G, cfg.S)

    # device copies ---------------------------------------------------------
    def dev_logits(self):
        return torch.from_numpy(self.logits).cuda()

    def dev_x(self):
        return to_device(wl.to_storage(self.x, self.cfg.dtype), self.cfg.dtype)

    def dev_hist_plan(self):
        return torch.from_numpy(np.ascontiguousarray(self.hist_plan, dtype=np.int32)).cuda()

    def dev_pred_idx(self):
        return None if self.pred_idx is None else torch.from_numpy(self.pred_idx).cuda()


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def to_host_f32(t):
    return t.detach().float().cpu().numpy()
