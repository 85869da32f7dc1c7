"""Seeded synthetic workloads for the MoE layer with dynamic expert duplication.

This module only *draws inputs*: router logits, activations, expert weights and
the two kinds of prediction the paper's strategies consume (a predicted
per-expert histogram for Distribution-Only Prediction, predicted per-token
expert ids for Token-to-Expert Prediction, Section 3.2).  It holds none of the
layer's arithmetic: anything that depends on the routing result (the true
histogram, the true top-k ids) is passed in by the caller.  Both the CPU oracle
tests and the GPU path draw from here so that they see identical numbers.

The paper measures on Mixtral 8x7B routing traces over MMLU / Alpaca Eval /
SST2 (Section 3.2.1, Table 1).  Neither the model nor the datasets are used
here; logits with a per-expert popularity bias stand in for them.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np

MODE_NONE = 0          # home placement only (no prediction baseline, Section 4)
MODE_DISTRIBUTION = 1  # Distribution-Only Prediction (Section 3.2.1)
MODE_TOKEN = 2         # Token-to-Expert Prediction (Section 3.2.2)


@dataclasses.dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int                 # tokens
    d: int                 # model width
    ffn: int               # expert hidden width
    E: int                 # experts
    k: int                 # experts per token
    G: int                 # virtual expert-parallel ranks
    S: int                 # expert slots per rank
    dtype: str             # "f32" or "bf16"
    mode: int              # MODE_*
    bias: str = "dirichlet"   # "dirichlet" or "zipf"
    alpha: float = 0.5     # Dirichlet concentration
    zipf_s: float = 1.2    # Zipf exponent
    sigma_pred: float = 0.0   # lognormal sigma of the predicted histogram (mode 1)
    acc: float = 1.0       # per-token prediction accuracy (mode 2)
    seed: int = 0
    c_max: int = 0         # max copies per expert; 0 -> G
    act: str = "swiglu"    # expert FFN form: "swiglu" (W1, W3, W2) or "relu" (W1, W2; W3 unused)

    @property
    def A(self) -> int:
        return self.T * self.k

    @property
    def nseg(self) -> int:
        return self.G * self.S

    @property
    def cmax(self) -> int:
        return self.c_max if self.c_max > 0 else self.G

    def replace(self, **kw) -> "MoEConfig":
        return dataclasses.replace(self, **kw)


def _cfg5(name, T, alpha, mode, seed):
    return MoEConfig(name, T=T, d=4096, ffn=1536, E=128, k=8, G=32, S=5, dtype="bf16",
                     mode=mode, alpha=alpha, sigma_pred=0.2, acc=0.85, seed=seed)


CONFIGS = {
    # tiny fp32 layer, distribution-only plan from the true histogram
    "cfg1_tiny_f32": MoEConfig("cfg1_tiny_f32", T=256, d=128, ffn=256, E=8, k=2, G=4, S=3,
                               dtype="f32", mode=MODE_DISTRIBUTION, alpha=0.5, sigma_pred=0.0, seed=0),
    # Mixtral-8x7B-shaped layer, distribution-only with a noisy histogram
    "cfg2_mixtral_dist": MoEConfig("cfg2_mixtral_dist", T=4096, d=4096, ffn=14336, E=8, k=2, G=8, S=2,
                                   dtype="bf16", mode=MODE_DISTRIBUTION, alpha=0.5, sigma_pred=0.2, seed=1),
    # same shape, token-to-expert prediction at 90 % accuracy
    "cfg3_mixtral_t2e": MoEConfig("cfg3_mixtral_t2e", T=4096, d=4096, ffn=14336, E=8, k=2, G=8, S=2,
                                  dtype="bf16", mode=MODE_TOKEN, alpha=0.5, acc=0.90, seed=2),
    # fine-grained MoE with Zipf popularity
    "cfg4_finegrained": MoEConfig("cfg4_finegrained", T=16384, d=2048, ffn=1408, E=64, k=6, G=16, S=5,
                                  dtype="bf16", mode=MODE_DISTRIBUTION, bias="zipf", zipf_s=1.2,
                                  sigma_pred=0.1, seed=3),
}
# skew / regime sweep: 3 Dirichlet alphas x 3 plan modes at prefill, plus decode
for _ai, _alpha in enumerate((0.1, 1.0, 10.0)):
    for _mode in (MODE_NONE, MODE_DISTRIBUTION, MODE_TOKEN):
        _n = f"cfg5_prefill_a{_alpha:g}_m{_mode}"
        CONFIGS[_n] = _cfg5(_n, 32768, _alpha, _mode, seed=4)
for _mode in (MODE_NONE, MODE_DISTRIBUTION, MODE_TOKEN):
    _n = f"cfg5_decode_m{_mode}"
    CONFIGS[_n] = _cfg5(_n, 128, 1.0, _mode, seed=4)

# Switch-Transformer-style layer: ReLU FFN, top-1 routing (Discussion, generality across
# model architectures); Switch-Base widths
CONFIGS["cfg6_switch_relu"] = MoEConfig("cfg6_switch_relu", T=16384, d=768, ffn=3072, E=64, k=1, G=8, S=10,
                                        dtype="bf16", mode=MODE_DISTRIBUTION, alpha=0.5, sigma_pred=0.2, seed=6,
                                        act="relu")

# LLaMA-MoE-style layer (Discussion; Appendix C): SwiGLU experts cut from a dense FFN, 16
# experts of width 11008 / 16 = 688, top-4
CONFIGS["cfg7_llama_moe"] = MoEConfig("cfg7_llama_moe", T=8192, d=4096, ffn=688, E=16, k=4, G=8, S=3,
                                      dtype="bf16", mode=MODE_DISTRIBUTION, alpha=0.5, sigma_pred=0.2, seed=7)

# a mid-size bf16 case the oracle can finish in full within seconds
CONFIGS["mid_bf16"] = MoEConfig("mid_bf16", T=512, d=512, ffn=1024, E=8, k=2, G=4, S=3,
                                dtype="bf16", mode=MODE_DISTRIBUTION, alpha=0.5, sigma_pred=0.2, seed=11)


def _rng(cfg: MoEConfig, stream: int, sub: int = 0) -> np.random.Generator:
    """Independent generator per (seed, purpose, sub-index)."""
    return np.random.default_rng([int(cfg.seed), int(stream), int(sub)])


# ---------------------------------------------------------------------------
# bf16 storage format helpers (format conversion only)
# ---------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(a: np.ndarray, dtype: str) -> np.ndarray:
    """Values as float32, rounded once to the storage dtype of the config."""
    a = np.asarray(a, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    return a


# ---------------------------------------------------------------------------
# router logits
# ---------------------------------------------------------------------------
def expert_popularity(cfg: MoEConfig) -> np.ndarray:
    """Per-expert popularity p (sums to 1) that biases the logits."""
    rng = _rng(cfg, 1)
    if cfg.bias == "dirichlet":
        p = rng.dirichlet(np.full(cfg.E, cfg.alpha, dtype=np.float64))
    elif cfg.bias == "zipf":
        ranks = np.arange(1, cfg.E + 1, dtype=np.float64)
        w = ranks ** (-cfg.zipf_s)
        w /= w.sum()
        p = np.empty(cfg.E, dtype=np.float64)
        p[rng.permutation(cfg.E)] = w
    else:
        raise ValueError(cfg.bias)
    return np.maximum(p, 1e-30)


def gen_logits(cfg: MoEConfig) -> np.ndarray:
    """logits[T, E] float32 = N(0, 1) + log popularity."""
    b = np.log(expert_popularity(cfg)).astype(np.float32)
    z = _rng(cfg, 2).standard_normal((cfg.T, cfg.E), dtype=np.float32)
    return (z + b[None, :]).astype(np.float32)


def gen_logits_batch(cfg: MoEConfig, batch: int) -> np.ndarray:
    """Batch ``batch`` of a stream of router logits with one fixed expert popularity
    (the i.i.d. setting of the Distribution-Only predictor): the bias of gen_logits,
    fresh N(0, 1) noise per batch.  Batch 0 is not gen_logits' batch."""
    b = np.log(expert_popularity(cfg)).astype(np.float32)
    z = _rng(cfg, 7, batch).standard_normal((cfg.T, cfg.E), dtype=np.float32)
    return (z + b[None, :]).astype(np.float32)


# ---------------------------------------------------------------------------
# activations and weights
# ---------------------------------------------------------------------------
def gen_x(cfg: MoEConfig) -> np.ndarray:
    """x[T, d] ~ N(0, 1), float32 values already rounded to the config's dtype."""
    x = _rng(cfg, 3).standard_normal((cfg.T, cfg.d), dtype=np.float32)
    return quantize(x, cfg.dtype)


def gen_expert_weights(cfg: MoEConfig, e: int):
    """(W1_e[d, ffn], W3_e[d, ffn], W2_e[ffn, d]) ~ N(0, 0.02), rounded to the dtype."""
    rng = _rng(cfg, 4, e)
    w1 = rng.standard_normal((cfg.d, cfg.ffn), dtype=np.float32) * np.float32(0.02)
    w3 = rng.standard_normal((cfg.d, cfg.ffn), dtype=np.float32) * np.float32(0.02)
    w2 = rng.standard_normal((cfg.ffn, cfg.d), dtype=np.float32) * np.float32(0.02)
    return quantize(w1, cfg.dtype), quantize(w3, cfg.dtype), quantize(w2, cfg.dtype)


def gen_weights_storage(cfg: MoEConfig, threads: int = 8):
    """All experts' weights in storage form: float32 arrays for "f32", uint16 bf16
    bit patterns for "bf16".  Shapes W1, W3: [E, d, ffn]; W2: [E, ffn, d]."""
    st = np.float32 if cfg.dtype == "f32" else np.uint16
    W1 = np.empty((cfg.E, cfg.d, cfg.ffn), dtype=st)
    W3 = np.empty((cfg.E, cfg.d, cfg.ffn), dtype=st)
    W2 = np.empty((cfg.E, cfg.ffn, cfg.d), dtype=st)

    def one(e):
        w1, w3, w2 = gen_expert_weights(cfg, e)
        if cfg.dtype == "f32":
            W1[e], W3[e], W2[e] = w1, w3, w2
        else:
            W1[e], W3[e], W2[e] = f32_to_bf16_bits(w1), f32_to_bf16_bits(w3), f32_to_bf16_bits(w2)

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(one, range(cfg.E)))
    return W1, W3, W2


def to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """float32 values (already representable) -> storage array for the device."""
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    return np.ascontiguousarray(a, dtype=np.float32)


def from_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return bf16_bits_to_f32(a)
    return np.asarray(a, dtype=np.float32)


# ---------------------------------------------------------------------------
# predictions (stand-ins for the paper's trained predictors, Section 3.2)
# ---------------------------------------------------------------------------
def gen_pred_hist(cfg: MoEConfig, hist_true: np.ndarray) -> np.ndarray:
    """Predicted per-expert counts for Distribution-Only Prediction: the true
    counts times lognormal(0, sigma) noise, rescaled to the same total and
    rounded by largest remainder (ties -> lowest expert) so the sum is exact."""
    n = np.asarray(hist_true, dtype=np.int64)
    total = int(n.sum())
    if cfg.sigma_pred <= 0.0 or total == 0:
        return n.astype(np.int32)
    zeta = _rng(cfg, 5).standard_normal(cfg.E)
    v = n.astype(np.float64) * np.exp(cfg.sigma_pred * zeta)
    if v.sum() <= 0:
        return n.astype(np.int32)
    v *= total / v.sum()
    base = np.floor(v).astype(np.int64)
    rem = total - int(base.sum())
    frac = v - base
    order = np.lexsort((np.arange(cfg.E), -frac))   # largest fraction first, ties -> lowest e
    base[order[:rem]] += 1
    assert int(base.sum()) == total
    return base.astype(np.int32)


def gen_pred_idx(cfg: MoEConfig, topk_idx_true: np.ndarray) -> np.ndarray:
    """Predicted expert ids for Token-to-Expert Prediction: with probability
    ``acc`` a token's row equals its true top-k row, otherwise it is k distinct
    experts drawn uniformly without replacement."""
    rng = _rng(cfg, 6)
    idx = np.asarray(topk_idx_true, dtype=np.int32).reshape(cfg.T, cfg.k)
    keep = rng.random(cfg.T) < cfg.acc
    # k distinct uniform ids per row: the k smallest of E random keys
    keys = rng.random((cfg.T, cfg.E))
    rand_rows = np.argsort(keys, axis=1, kind="stable")[:, :cfg.k].astype(np.int32)
    return np.where(keep[:, None], idx, rand_rows).astype(np.int32)


def gen_pred_idx_concentrated(cfg: MoEConfig, topk_idx_true: np.ndarray, target_expert: np.ndarray) -> np.ndarray:
    """Predicted ids whose errors all fall on a chosen set of experts (the pessimistic case of
    Section 3.3: every misprediction lands on one device when the set is that device's home
    experts).  Rows equal the true rows except that, token by token in ascending order, the
    entries whose true expert is in ``target_expert`` (bool [E]) are replaced by the lowest
    expert ids that are neither in the token's true row nor already used in the row, until
    (1 - acc) * A entries have been replaced or no such entry is left."""
    idx = np.asarray(topk_idx_true, dtype=np.int32).reshape(cfg.T, cfg.k)
    target = np.asarray(target_expert, dtype=bool)
    budget = int(round((1.0 - cfg.acc) * cfg.A))
    out = idx.copy()
    for t in range(cfg.T):
        if budget <= 0:
            break
        hit = np.nonzero(target[idx[t]])[0]
        if hit.size == 0:
            continue
        free = [e for e in range(cfg.E) if e not in set(idx[t].tolist())]
        for n, j in enumerate(hit[:budget]):
            if n >= len(free):
                break
            out[t, j] = free[n]
            budget -= 1
    return out

