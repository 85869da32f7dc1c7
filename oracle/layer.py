"""Oracle: one pass of the whole MoE layer with expert duplication
(test infrastructure, CPU only).

Order of the steps follows the single-layer flow of Figure 3 restricted to the
FFN side: route (gate top-k) -> per-expert histogram -> duplication plan from the
prediction (Algorithm 1) -> dispatch/permutation -> expert FFN -> combine.
"""
import numpy as np

from .routing import route_topk
from .histogram import histogram
from .plan import plan_duplicates, MODE_TOKEN
from .permute import permute
from .ffn import grouped_ffn
from .combine import combine


def moe_layer(mode, logits, x, W1, W3, W2, k, G, S, c_max, hist_pred=None, pred_idx=None):
    """Returns a dict with every intermediate.  For mode 1 ``hist_pred`` is the
    predicted histogram; for mode 2 ``pred_idx[T, k]`` are the predicted ids and
    the plan is built from their histogram; mode 0 ignores both."""
    logits = np.asarray(logits)
    T, E = logits.shape
    idx, w = route_topk(logits, k)
    hist = histogram(idx, E)
    if mode == MODE_TOKEN:
        hist_plan = histogram(pred_idx, E)
    elif hist_pred is not None:
        hist_plan = np.asarray(hist_pred)
    else:
        hist_plan = hist
    plan = plan_duplicates(mode, hist_plan, E, G, S, c_max)
    perm = permute(mode, x, idx, pred_idx, hist, hist_plan, plan.slot_expert, plan.slot_quota, E, G, S)
    y_perm = grouped_ffn(perm["x_perm"], perm["seg_offsets"], plan.slot_expert, W1, W3, W2)
    out = combine(y_perm, perm["row_of_assign"], w, T, k)
    return dict(topk_idx=idx, topk_w=w, hist=hist, hist_plan=hist_plan, plan=plan, perm=perm,
                y_perm=y_perm, out=out)
