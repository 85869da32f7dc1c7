"""One MoE FFN layer with dynamic expert duplication, as a sequence of C-ABI calls.

``MoELayer`` owns the device buffers (allocated once through torch) and runs the
path route -> histogram -> duplication plan -> permute -> grouped FFN -> combine
(the FFN side of the single-layer flow in Figure 3) with no host synchronisation
between the calls.  Every step runs inside libmoegps; this file only sequences
the calls and keeps the buffers.
"""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as B
from .workloads import MODE_DISTRIBUTION, MODE_NONE, MODE_TOKEN, MoEConfig


def torch_dtype(cfg: MoEConfig):
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def to_device(a: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """Storage array from ``workloads`` (float32, or uint16 bf16 bit patterns) -> GPU tensor."""
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


class MoELayer:
    def __init__(self, cfg: MoEConfig, device="cuda", fused_gather: bool = False, fused_weights: bool = False):
        """fused_gather: gather the token rows inside the first FFN product
        (moe_grouped_ffn_gather) instead of materialising x_perm in moe_permute.
        fused_weights (implies fused_gather): the second product also applies the gate weights
        (moe_grouped_ffn_fused) and moe_combine only adds the k rows of a token."""
        self.cfg = cfg
        self.fused_weights = fused_weights
        fused_gather = fused_gather or fused_weights
        self.fused_gather = fused_gather
        self.dev = torch.device(device)
        c = cfg
        dt = torch_dtype(c)
        i32 = dict(dtype=torch.int32, device=self.dev)
        self.topk_idx = torch.empty((c.T, c.k), **i32)
        self.topk_w = torch.empty((c.T, c.k), dtype=torch.float32, device=self.dev)
        self.hist = torch.empty(c.E, **i32)
        self.hist_plan = torch.empty(c.E, **i32)
        self.slot_expert = torch.empty(c.nseg, **i32)
        self.slot_quota = torch.empty(c.nseg, **i32)
        self.rank_load_pred = torch.empty(c.G, **i32)
        self.n_iters = torch.empty(1, **i32)
        self.perm = dict(
            seg_offsets=torch.empty(c.nseg + 1, **i32),
            row_of_assign=torch.empty(c.A, **i32),
            assign_of_row=torch.empty(c.A, **i32),
            x_perm=None if fused_gather else torch.empty((c.A, c.d), dtype=dt, device=self.dev),
            rank_load=torch.empty(c.G, **i32),
        )
        self.y_perm = torch.zeros((c.A, c.d), dtype=dt, device=self.dev)
        self.out = torch.empty((c.T, c.d), dtype=dt, device=self.dev)
        dcode = B.MOE_DTYPE_F32 if c.dtype == "f32" else B.MOE_DTYPE_BF16
        self.ws_perm = torch.empty(max(256, B.moe_permute_workspace_bytes(c.T, c.E, c.k, c.G, c.S)),
                                   dtype=torch.uint8, device=self.dev)
        self.ws_ffn = torch.empty(max(256, B.moe_grouped_ffn_workspace_bytes(c.A, c.d, c.ffn, c.nseg, dcode)),
                                  dtype=torch.uint8, device=self.dev)
        self.packed: Optional[torch.Tensor] = None

    def set_weights(self, W1: torch.Tensor, W3: Optional[torch.Tensor], W2: torch.Tensor) -> None:
        """One-off repack of the (static) expert weights; the ReLU form has no W3."""
        if self.cfg.act == "relu":
            if self.fused_gather:
                raise B.MoeGpsError("the fused row gather is built for the SwiGLU form only")
            self.packed = B.moe_pack_weights_relu(W1, W2)
        else:
            self.packed = B.moe_pack_weights(W1, W3, W2)

    # individual steps (each is exactly one C-ABI call) ---------------------
    def route(self, logits):
        B.moe_route_topk(logits, self.cfg.k, out=(self.topk_idx, self.topk_w))

    def histogram(self):
        B.moe_histogram(self.topk_idx, self.cfg.E, out=self.hist)

    def plan(self, mode, hist_pred: Optional[torch.Tensor], pred_idx: Optional[torch.Tensor]):
        c = self.cfg
        if mode == MODE_TOKEN:
            B.moe_histogram(pred_idx, c.E, out=self.hist_plan)
            hp = self.hist_plan
        elif mode == MODE_DISTRIBUTION:
            hp = hist_pred
        else:
            hp = self.hist
        self._hp = hp
        B.moe_plan_duplicates(mode, hp, c.G, c.S, c.cmax,
                              out=(self.slot_expert, self.slot_quota, self.rank_load_pred, self.n_iters))

    def permute(self, mode, x, pred_idx):
        c = self.cfg
        self._x = x
        B.moe_permute(mode, x, self.topk_idx, pred_idx if mode == MODE_TOKEN else None, self.hist, self._hp,
                      self.slot_expert, self.slot_quota, c.E, c.G, c.S, workspace=self.ws_perm, out=self.perm)

    def ffn(self, seg_begin=0, seg_end=None):
        c = self.cfg
        if self.packed is None:
            raise B.MoeGpsError("set_weights() first")
        if self.fused_gather:
            B.moe_grouped_ffn_gather(self._x, self.perm["assign_of_row"], c.k, self.perm["seg_offsets"],
                                     self.slot_expert, self.packed, c.E, c.ffn, seg_begin, seg_end,
                                     workspace=self.ws_ffn, out=self.y_perm,
                                     topk_w=self.topk_w if self.fused_weights else None)
        else:
            B.moe_grouped_ffn(self.perm["x_perm"], self.perm["seg_offsets"], self.slot_expert, self.packed, c.E,
                              c.ffn, seg_begin, seg_end, workspace=self.ws_ffn, out=self.y_perm,
                              relu=(c.act == "relu"))

    def combine(self):
        c = self.cfg
        B.moe_combine(self.y_perm, self.perm["row_of_assign"], None if self.fused_weights else self.topk_w, c.T, c.k,
                      out=self.out)

    # the whole path -----------------------------------------------------------
    def step(self, logits: torch.Tensor, x: torch.Tensor, hist_pred: Optional[torch.Tensor] = None,
             pred_idx: Optional[torch.Tensor] = None, mode: Optional[int] = None) -> torch.Tensor:
        mode = self.cfg.mode if mode is None else mode
        self.route(logits)
        self.histogram()
        self.plan(mode, hist_pred, pred_idx)
        self.permute(mode, x, pred_idx)
        self.ffn()
        self.combine()
        return self.out

    def capture(self, logits: torch.Tensor, x: torch.Tensor, hist_pred: Optional[torch.Tensor] = None,
                pred_idx: Optional[torch.Tensor] = None, mode: Optional[int] = None):
        """Records one whole step into a HIP graph and returns it (``graph.replay()`` then runs
        the step again on whatever the same input tensors hold by then; the result is in
        ``self.out``).  Every call of the library only enqueues kernels on the current stream and
        this object owns all buffers, so the step captures as it is: no allocation, no host
        synchronisation, no memset nodes.  One eager step runs first (it sets the kernels' LDS
        attribute, which is not a stream operation)."""
        self.step(logits, x, hist_pred=hist_pred, pred_idx=pred_idx, mode=mode)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.step(logits, x, hist_pred=hist_pred, pred_idx=pred_idx, mode=mode)
        return graph

    def comm_report(self, mode=None, pred_idx: Optional[torch.Tensor] = None, link_GBs: float = 153.6) -> dict:
        """Rows (and bytes) that would cross the emulated ranks at dispatch and combine for the
        last permutation (one C-ABI call + host read-back, off the timed path), next to the
        closed forms of the paper's Background: (G-1)/G of all rows move when the placement is
        balanced, and the busiest receiver gets (G-1)/G^2 * (max rank load / mean rank load).
        ``time_us`` models a full mesh of point-to-point links (one per ordered pair of ranks,
        ``link_GBs`` each way): the slowest pair decides."""
        c = self.cfg
        mode = c.mode if mode is None else mode
        disp, comb = B.moe_comm_matrix(mode, self.topk_idx, pred_idx if mode == MODE_TOKEN else None,
                                       self.perm["row_of_assign"], self.perm["seg_offsets"], c.G, c.S)
        disp = disp.cpu().numpy().astype(np.int64)
        comb = comb.cpu().numpy().astype(np.int64)
        row_bytes = c.d * (2 if c.dtype == "bf16" else 4)
        A = int(disp.sum())
        load = disp.sum(axis=0)

        def side(m):
            off = m - np.diag(np.diag(m))
            return dict(crossing_rows=int(off.sum()), crossing_frac=float(off.sum() / A) if A else 0.0,
                        max_inbound_rows=int(off.sum(axis=0).max()), max_outbound_rows=int(off.sum(axis=1).max()),
                        max_pair_rows=int(off.max()), bytes=int(off.sum()) * row_bytes,
                        time_us=float(off.max() * row_bytes / (link_GBs * 1e9) * 1e6))

        rank_skew = float(load.max() * c.G / A) if A else 0.0
        return dict(mode=mode, dispatch=side(disp), combine=side(comb),
                    balanced_crossing_frac=(c.G - 1) / c.G,
                    bottleneck_inbound_frac_model=(c.G - 1) * rank_skew / c.G**2,
                    bottleneck_inbound_frac=float((disp.sum(axis=0) - np.diag(disp)).max() / A) if A else 0.0,
                    dispatch_matrix=disp.tolist() if c.G <= 8 else None)

    def load_report(self) -> dict:
        """Host read-back (off the timed path): per-rank rows, makespan, imbalance and
        skewness (most popular expert's tokens / average tokens per expert)."""
        c = self.cfg
        rank_load = self.perm["rank_load"].cpu().numpy().astype(np.int64)
        hist = self.hist.cpu().numpy().astype(np.int64)
        A = int(hist.sum())
        return dict(
            rank_load=rank_load.tolist(),
            makespan=int(rank_load.max()) if rank_load.size else 0,
            imbalance=float(rank_load.max() * c.G / A) if A else 0.0,
            skewness=float(hist.max() * c.E / A) if A else 0.0,
            n_iters=int(self.n_iters.item()),
            replicas=int((self.slot_expert.cpu().numpy() >= 0).sum() - c.E),
        )
