"""Oracle: top-k gating (test infrastructure, CPU only).

Background section, "each token is routed to its top-1 experts ... the general
concepts apply to ... top-K experts": the token->expert map f of Algorithm 1's
input.  The paper fixes only which experts a token goes to; two readings are
taken where it is silent:
  * ties between equal logits go to the lowest expert index;
  * gate weights are a softmax over the k selected logits (the convention of the
    Mixtral-style model the paper evaluates).
"""
import numpy as np


def route_topk(logits: np.ndarray, k: int):
    """Return (topk_idx[T, k] int32, topk_w[T, k] float64).

    For every token the experts are ordered by (logit descending, index
    ascending) and the first k are taken, in that order.  Weights are
    exp(l_j - l_0) / sum_i exp(l_i - l_0) over the k selected logits, in fp64.
    """
    logits = np.asarray(logits)
    T, E = logits.shape
    assert 1 <= k <= E
    # a stable sort of the negated row puts larger logits first and keeps equal
    # logits in ascending index order
    order = np.argsort(-logits, axis=1, kind="stable")
    idx = order[:, :k].astype(np.int32)
    sel = np.take_along_axis(logits.astype(np.float64), idx.astype(np.int64), axis=1)
    ex = np.exp(sel - sel[:, :1])
    w = ex / ex.sum(axis=1, keepdims=True)
    return idx, w
