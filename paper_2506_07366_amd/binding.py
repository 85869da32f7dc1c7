"""Thin ctypes binding over libmoegps.so (argument marshalling only).

Every function takes torch tensors that already live on the GPU, checks dtype /
contiguity / device, passes raw device pointers and the current HIP stream to the
C ABI declared in ``include/moegps.h`` and raises ``MoeGpsError`` on a non-zero
return code.  There is no CPU fallback: if the shared library has not been built
the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoegps.so")

MOE_DTYPE_F32 = 0
MOE_DTYPE_BF16 = 1
MODE_NONE, MODE_DISTRIBUTION, MODE_TOKEN = 0, 1, 2

EXPORTS = [
    "moe_strerror", "moe_last_hip_error", "moe_abi_version", "moe_route_topk", "moe_histogram",
    "moe_plan_duplicates", "moe_permute_workspace_bytes", "moe_permute", "moe_permute_static",
    "moe_packed_weights_bytes",
    "moe_pack_weights", "moe_grouped_ffn_workspace_bytes", "moe_grouped_ffn", "moe_grouped_ffn_gather",
    "moe_grouped_ffn_fused", "moe_grouped_ffn_set_option", "moe_grouped_ffn_time_next_call",
    "moe_combine", "moe_comm_matrix", "moe_predictor_update", "moe_predictor_predict",
    "moe_packed_weights_relu_bytes", "moe_pack_weights_relu", "moe_grouped_ffn_relu",
]


class MoeGpsError(RuntimeError):
    pass


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load libmoegps.so and declare the argument types of every entry point."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or os.environ.get("MOEGPS_LIB") or LIB_PATH
    if not os.path.exists(p):
        raise MoeGpsError(
            f"{p} is missing: build it first with `python -m paper_2506_07366_amd.build` "
            "(the HIP library is required, there is no fallback path)")
    lib = ctypes.CDLL(p)
    c_int, c_i64, c_sz, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_size_t, ctypes.c_void_p
    lib.moe_strerror.restype = ctypes.c_char_p
    lib.moe_strerror.argtypes = [c_int]
    lib.moe_last_hip_error.restype = c_int
    lib.moe_last_hip_error.argtypes = []
    lib.moe_abi_version.restype = c_int
    lib.moe_abi_version.argtypes = []
    lib.moe_route_topk.restype = c_int
    lib.moe_route_topk.argtypes = [vp, c_int, c_int, c_int, vp, vp, vp]
    lib.moe_histogram.restype = c_int
    lib.moe_histogram.argtypes = [vp, c_i64, c_int, vp, vp]
    lib.moe_plan_duplicates.restype = c_int
    lib.moe_plan_duplicates.argtypes = [c_int, vp, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp]
    lib.moe_permute_workspace_bytes.restype = c_sz
    lib.moe_permute_workspace_bytes.argtypes = [c_int] * 5
    lib.moe_permute.restype = c_int
    lib.moe_permute.argtypes = [c_int, vp, c_int, c_int, c_int, c_int, c_int, c_int, c_int,
                                vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, c_sz, vp]
    lib.moe_permute_static.restype = c_int
    lib.moe_permute_static.argtypes = lib.moe_permute.argtypes[:20] + [vp]
    lib.moe_packed_weights_bytes.restype = c_sz
    lib.moe_packed_weights_bytes.argtypes = [c_int] * 4
    lib.moe_pack_weights.restype = c_int
    lib.moe_pack_weights.argtypes = [vp, vp, vp, c_int, c_int, c_int, c_int, vp, vp]
    lib.moe_grouped_ffn_workspace_bytes.restype = c_sz
    lib.moe_grouped_ffn_workspace_bytes.argtypes = [c_i64, c_int, c_int, c_int, c_int]
    lib.moe_grouped_ffn.restype = c_int
    lib.moe_grouped_ffn.argtypes = [vp, c_int, c_i64, c_int, c_int, c_int, vp, vp, c_int, c_int, c_int,
                                    vp, vp, vp, c_sz, vp]
    lib.moe_packed_weights_relu_bytes.restype = c_sz
    lib.moe_packed_weights_relu_bytes.argtypes = [c_int] * 4
    lib.moe_pack_weights_relu.restype = c_int
    lib.moe_pack_weights_relu.argtypes = [vp, vp, c_int, c_int, c_int, c_int, vp, vp]
    lib.moe_grouped_ffn_relu.restype = c_int
    lib.moe_grouped_ffn_relu.argtypes = lib.moe_grouped_ffn.argtypes
    lib.moe_grouped_ffn_gather.restype = c_int
    lib.moe_grouped_ffn_gather.argtypes = [vp, c_int, c_int, c_int, vp, c_int, c_int, c_int, vp, vp, c_int, c_int,
                                           c_int, vp, vp, vp, c_sz, vp]
    lib.moe_grouped_ffn_fused.restype = c_int
    lib.moe_grouped_ffn_fused.argtypes = [vp, c_int, c_int, c_int, vp, vp, c_int, c_int, c_int, vp, vp, c_int, c_int,
                                          c_int, vp, vp, vp, c_sz, vp]
    lib.moe_grouped_ffn_set_option.restype = c_int
    lib.moe_grouped_ffn_set_option.argtypes = [c_int, c_int]
    lib.moe_grouped_ffn_time_next_call.restype = c_int
    lib.moe_grouped_ffn_time_next_call.argtypes = [ctypes.POINTER(vp)]
    lib.moe_combine.restype = c_int
    lib.moe_combine.argtypes = [vp, c_int, c_int, c_int, c_int, vp, vp, vp, vp]
    lib.moe_predictor_update.restype = c_int
    lib.moe_predictor_update.argtypes = [vp, c_int, vp, vp]
    lib.moe_predictor_predict.restype = c_int
    lib.moe_predictor_predict.argtypes = [vp, c_int, c_i64, vp, vp]
    lib.moe_comm_matrix.restype = c_int
    lib.moe_comm_matrix.argtypes = [c_int, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp, vp, vp]
    if path is None:
        _lib = lib
    return lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        lib = load_library()
        msg = lib.moe_strerror(rc).decode()
        extra = f" (hipError {lib.moe_last_hip_error()})" if rc == -4 else ""
        raise MoeGpsError(f"{what}: {msg}{extra}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _need(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise MoeGpsError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise MoeGpsError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise MoeGpsError(f"{name} must be contiguous")
    return t


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MOE_DTYPE_F32
    if t.dtype == torch.bfloat16:
        return MOE_DTYPE_BF16
    raise MoeGpsError(f"unsupported dtype {t.dtype}")


def moe_route_topk(logits: torch.Tensor, k: int, out=None):
    """``out``: optional (topk_idx, topk_w) to write into."""
    lib = load_library()
    _need(logits, torch.float32, "logits")
    T, E = logits.shape
    if out is None:
        idx = torch.empty((T, k), dtype=torch.int32, device=logits.device)
        w = torch.empty((T, k), dtype=torch.float32, device=logits.device)
    else:
        idx, w = out
        _need(idx, torch.int32, "topk_idx")
        _need(w, torch.float32, "topk_w")
    _check(lib.moe_route_topk(_ptr(logits), T, E, k, _ptr(idx), _ptr(w), _stream()), "moe_route_topk")
    return idx, w


def moe_histogram(idx: torch.Tensor, E: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    lib = load_library()
    _need(idx, torch.int32, "idx")
    hist = out if out is not None else torch.empty(E, dtype=torch.int32, device=idx.device)
    _check(lib.moe_histogram(_ptr(idx), idx.numel(), E, _ptr(hist), _stream()), "moe_histogram")
    return hist


def moe_plan_duplicates(mode: int, hist_pred: torch.Tensor, G: int, S: int, c_max: int, out=None):
    """``out``: optional (slot_expert, slot_quota, rank_load_pred, n_iters) to write into."""
    lib = load_library()
    _need(hist_pred, torch.int32, "hist_pred")
    E = hist_pred.numel()
    dev = hist_pred.device
    if out is None:
        slot_expert = torch.empty(G * S, dtype=torch.int32, device=dev)
        slot_quota = torch.empty(G * S, dtype=torch.int32, device=dev)
        rank_load_pred = torch.empty(G, dtype=torch.int32, device=dev)
        n_iters = torch.empty(1, dtype=torch.int32, device=dev)
    else:
        slot_expert, slot_quota, rank_load_pred, n_iters = out
        for name, t in (("slot_expert", slot_expert), ("slot_quota", slot_quota),
                        ("rank_load_pred", rank_load_pred), ("n_iters", n_iters)):
            _need(t, torch.int32, name)
    _check(lib.moe_plan_duplicates(mode, _ptr(hist_pred), E, G, S, c_max, _ptr(slot_expert), _ptr(slot_quota),
                                   _ptr(rank_load_pred), _ptr(n_iters), _stream()), "moe_plan_duplicates")
    return slot_expert, slot_quota, rank_load_pred, n_iters


def moe_permute_workspace_bytes(T: int, E: int, k: int, G: int, S: int) -> int:
    return int(load_library().moe_permute_workspace_bytes(T, E, k, G, S))


def moe_permute(mode: int, x: Optional[torch.Tensor], topk_idx: torch.Tensor, pred_idx: Optional[torch.Tensor],
                hist_true: Optional[torch.Tensor], hist_pred: Optional[torch.Tensor],
                slot_expert: torch.Tensor, slot_quota: torch.Tensor, E: int, G: int, S: int,
                workspace: Optional[torch.Tensor] = None, copy_rows: bool = True, out: Optional[dict] = None,
                static_scratch: bool = False):
    """Returns dict(seg_offsets, row_of_assign, assign_of_row, x_perm, rank_load).
    ``static_scratch=True`` calls moe_permute_static (no workspace; pass ``out`` to allocate nothing at all)."""
    lib = load_library()
    _need(topk_idx, torch.int32, "topk_idx")
    T, k = topk_idx.shape
    dev = topk_idx.device
    if x is not None:
        if not x.is_cuda or not x.is_contiguous():
            raise MoeGpsError("x must be a contiguous GPU tensor")
        d = x.shape[1]
        dt = dtype_code(x)
    else:
        d, dt = 4, MOE_DTYPE_F32
    for name, t in (("pred_idx", pred_idx), ("hist_true", hist_true), ("hist_pred", hist_pred),
                    ("slot_expert", slot_expert), ("slot_quota", slot_quota)):
        if t is not None:
            _need(t, torch.int32, name)
    A = T * k
    if out is None:
        out = dict(
            seg_offsets=torch.empty(G * S + 1, dtype=torch.int32, device=dev),
            row_of_assign=torch.empty(A, dtype=torch.int32, device=dev),
            assign_of_row=torch.empty(A, dtype=torch.int32, device=dev),
            x_perm=(torch.empty((A, d), dtype=x.dtype, device=dev) if (x is not None and copy_rows) else None),
            rank_load=torch.empty(G, dtype=torch.int32, device=dev),
        )
    if static_scratch:
        # the variant that allocates nothing: scratch is the library's own fixed device array
        _check(lib.moe_permute_static(mode, _ptr(x), dt, T, d, E, k, G, S, _ptr(topk_idx), _ptr(pred_idx),
                                      _ptr(hist_true), _ptr(hist_pred), _ptr(slot_expert), _ptr(slot_quota),
                                      _ptr(out["seg_offsets"]), _ptr(out["row_of_assign"]),
                                      _ptr(out["assign_of_row"]), _ptr(out["x_perm"]), _ptr(out["rank_load"]),
                                      _stream()), "moe_permute_static")
        return out
    need = moe_permute_workspace_bytes(T, E, k, G, S)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    _check(lib.moe_permute(mode, _ptr(x), dt, T, d, E, k, G, S, _ptr(topk_idx), _ptr(pred_idx), _ptr(hist_true),
                           _ptr(hist_pred), _ptr(slot_expert), _ptr(slot_quota), _ptr(out["seg_offsets"]),
                           _ptr(out["row_of_assign"]), _ptr(out["assign_of_row"]), _ptr(out["x_perm"]),
                           _ptr(out["rank_load"]), _ptr(workspace), workspace.numel(), _stream()), "moe_permute")
    return out


def moe_packed_weights_bytes(E: int, d: int, ffn: int, dtype: int) -> int:
    return int(load_library().moe_packed_weights_bytes(E, d, ffn, dtype))


def moe_pack_weights(W1: torch.Tensor, W3: torch.Tensor, W2: torch.Tensor) -> torch.Tensor:
    lib = load_library()
    dt = dtype_code(W1)
    for name, t in (("W1", W1), ("W3", W3), ("W2", W2)):
        _need(t, W1.dtype, name)
    E, d, ffn = W1.shape
    if tuple(W3.shape) != (E, d, ffn) or tuple(W2.shape) != (E, ffn, d):
        raise MoeGpsError("weight shapes must be W1,W3 [E,d,ffn] and W2 [E,ffn,d]")
    packed = torch.empty(moe_packed_weights_bytes(E, d, ffn, dt), dtype=torch.uint8, device=W1.device)
    _check(lib.moe_pack_weights(_ptr(W1), _ptr(W3), _ptr(W2), dt, E, d, ffn, _ptr(packed), _stream()),
           "moe_pack_weights")
    return packed


def moe_grouped_ffn_workspace_bytes(A: int, d: int, ffn: int, nseg: int, dtype: int) -> int:
    return int(load_library().moe_grouped_ffn_workspace_bytes(A, d, ffn, nseg, dtype))


def moe_pack_weights_relu(W1: torch.Tensor, W2: torch.Tensor) -> torch.Tensor:
    """Packed weights of the ReLU form of the FFN (W1 [E, d, ffn], W2 [E, ffn, d])."""
    lib = load_library()
    dt = dtype_code(W1)
    _need(W2, W1.dtype, "W2")
    E, d, ffn = W1.shape
    if tuple(W2.shape) != (E, ffn, d):
        raise MoeGpsError("weight shapes must be W1 [E,d,ffn] and W2 [E,ffn,d]")
    packed = torch.empty(int(lib.moe_packed_weights_relu_bytes(E, d, ffn, dt)), dtype=torch.uint8, device=W1.device)
    _check(lib.moe_pack_weights_relu(_ptr(W1), _ptr(W2), dt, E, d, ffn, _ptr(packed), _stream()),
           "moe_pack_weights_relu")
    return packed


def moe_grouped_ffn(x_perm: torch.Tensor, seg_offsets: torch.Tensor, slot_expert: torch.Tensor, packed: torch.Tensor,
                    E: int, ffn: int, seg_begin: int = 0, seg_end: Optional[int] = None,
                    workspace: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                    relu: bool = False) -> torch.Tensor:
    """``relu=True`` calls moe_grouped_ffn_relu (``packed`` from moe_pack_weights_relu)."""
    lib = load_library()
    dt = dtype_code(x_perm)
    if not x_perm.is_contiguous() or not x_perm.is_cuda:
        raise MoeGpsError("x_perm must be a contiguous GPU tensor")
    _need(seg_offsets, torch.int32, "seg_offsets")
    _need(slot_expert, torch.int32, "slot_expert")
    A, d = x_perm.shape
    nseg = slot_expert.numel()
    if seg_end is None:
        seg_end = nseg
    y = out if out is not None else torch.zeros_like(x_perm)
    need = moe_grouped_ffn_workspace_bytes(A, d, ffn, nseg, dt)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x_perm.device)
    fn = lib.moe_grouped_ffn_relu if relu else lib.moe_grouped_ffn
    _check(fn(_ptr(x_perm), dt, A, d, ffn, E, _ptr(seg_offsets), _ptr(slot_expert), nseg, seg_begin, seg_end,
              _ptr(packed), _ptr(y), _ptr(workspace), workspace.numel(), _stream()),
           "moe_grouped_ffn_relu" if relu else "moe_grouped_ffn")
    return y


def moe_grouped_ffn_gather(x: torch.Tensor, assign_of_row: torch.Tensor, k: int, seg_offsets: torch.Tensor,
                           slot_expert: torch.Tensor, packed: torch.Tensor, E: int, ffn: int, seg_begin: int = 0,
                           seg_end: Optional[int] = None, workspace: Optional[torch.Tensor] = None,
                           out: Optional[torch.Tensor] = None, topk_w: Optional[torch.Tensor] = None) -> torch.Tensor:
    """FFN with the row gather fused into the first product (no x_perm).  With ``topk_w``
    (moe_grouped_ffn_fused) the rows of the result are also multiplied by their gate weights."""
    lib = load_library()
    dt = dtype_code(x)
    if not x.is_contiguous() or not x.is_cuda:
        raise MoeGpsError("x must be a contiguous GPU tensor")
    _need(assign_of_row, torch.int32, "assign_of_row")
    _need(seg_offsets, torch.int32, "seg_offsets")
    _need(slot_expert, torch.int32, "slot_expert")
    T, d = x.shape
    A = T * k
    nseg = slot_expert.numel()
    if seg_end is None:
        seg_end = nseg
    y = out if out is not None else torch.zeros((A, d), dtype=x.dtype, device=x.device)
    need = moe_grouped_ffn_workspace_bytes(A, d, ffn, nseg, dt)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if topk_w is not None:
        _need(topk_w, torch.float32, "topk_w")
        _check(lib.moe_grouped_ffn_fused(_ptr(x), dt, T, k, _ptr(assign_of_row), _ptr(topk_w), d, ffn, E,
                                         _ptr(seg_offsets), _ptr(slot_expert), nseg, seg_begin, seg_end, _ptr(packed),
                                         _ptr(y), _ptr(workspace), workspace.numel(), _stream()),
               "moe_grouped_ffn_fused")
        return y
    _check(lib.moe_grouped_ffn_gather(_ptr(x), dt, T, k, _ptr(assign_of_row), d, ffn, E, _ptr(seg_offsets),
                                      _ptr(slot_expert), nseg, seg_begin, seg_end, _ptr(packed), _ptr(y),
                                      _ptr(workspace), workspace.numel(), _stream()), "moe_grouped_ffn_gather")
    return y


FFN_OPT_TILE1, FFN_OPT_TILE2, FFN_OPT_SPLIT_K, FFN_OPT_GROUP_N = 0, 1, 2, 3


def moe_grouped_ffn_set_option(option: int, value: int) -> None:
    """Process-wide override of an automatic choice inside the grouped FFN (tests, experiments)."""
    _check(load_library().moe_grouped_ffn_set_option(option, value), "moe_grouped_ffn_set_option")


def moe_combine(y_perm: torch.Tensor, row_of_assign: torch.Tensor, topk_w: Optional[torch.Tensor], T: int, k: int,
                out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """``topk_w=None``: the rows already carry their gate weights and are only added."""
    lib = load_library()
    dt = dtype_code(y_perm)
    _need(row_of_assign, torch.int32, "row_of_assign")
    if topk_w is not None:
        _need(topk_w, torch.float32, "topk_w")
    d = y_perm.shape[1]
    if out is None:
        out = torch.empty((T, d), dtype=y_perm.dtype, device=y_perm.device)
    _check(lib.moe_combine(_ptr(y_perm), dt, T, d, k, _ptr(row_of_assign), _ptr(topk_w), _ptr(out), _stream()),
           "moe_combine")
    return out


def moe_comm_matrix(mode: int, topk_idx: torch.Tensor, pred_idx: Optional[torch.Tensor],
                    row_of_assign: torch.Tensor, seg_offsets: torch.Tensor, G: int, S: int):
    """Returns (dispatch, combine): int32 [G, G] counts of rows by [source rank, destination rank]."""
    lib = load_library()
    _need(topk_idx, torch.int32, "topk_idx")
    _need(row_of_assign, torch.int32, "row_of_assign")
    _need(seg_offsets, torch.int32, "seg_offsets")
    if pred_idx is not None:
        _need(pred_idx, torch.int32, "pred_idx")
    T, k = topk_idx.shape
    dispatch = torch.empty((G, G), dtype=torch.int32, device=topk_idx.device)
    combine = torch.empty((G, G), dtype=torch.int32, device=topk_idx.device)
    _check(lib.moe_comm_matrix(mode, T, k, G, S, _ptr(topk_idx), _ptr(pred_idx), _ptr(row_of_assign),
                               _ptr(seg_offsets), _ptr(dispatch), _ptr(combine), _stream()), "moe_comm_matrix")
    return dispatch, combine


def moe_predictor_update(hist: torch.Tensor, counts: torch.Tensor) -> None:
    """counts[e] += hist[e] (counts: int64 [E], zeroed by the caller before the first batch)."""
    lib = load_library()
    _need(hist, torch.int32, "hist")
    _need(counts, torch.int64, "counts")
    if hist.numel() != counts.numel():
        raise MoeGpsError("hist and counts must have one entry per expert")
    _check(lib.moe_predictor_update(_ptr(hist), hist.numel(), _ptr(counts), _stream()), "moe_predictor_update")


def moe_predictor_predict(counts: torch.Tensor, A_next: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Predicted histogram (int32 [E], sums to A_next) from the cumulative counts."""
    lib = load_library()
    _need(counts, torch.int64, "counts")
    if out is None:
        out = torch.empty(counts.numel(), dtype=torch.int32, device=counts.device)
    _check(lib.moe_predictor_predict(_ptr(counts), counts.numel(), A_next, _ptr(out), _stream()),
           "moe_predictor_predict")
    return out


def moe_grouped_ffn_time_next_call(events) -> None:
    """``events``: four recorded-once ``torch.cuda.Event(enable_timing=True)``; the next
    moe_grouped_ffn call on this thread records them around its two products."""
    lib = load_library()
    if events is None:
        _check(lib.moe_grouped_ffn_time_next_call(None), "moe_grouped_ffn_time_next_call")
        return
    arr = (ctypes.c_void_p * 4)(*[ctypes.c_void_p(e.cuda_event) for e in events])
    _check(lib.moe_grouped_ffn_time_next_call(arr), "moe_grouped_ffn_time_next_call")
