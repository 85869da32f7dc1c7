"""The C-ABI library loads and exports every symbol the header declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "moegps.h")


def declared_symbols():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", src)))


def test_header_declares_the_path():
    syms = declared_symbols()
    for name in ["moe_route_topk", "moe_histogram", "moe_plan_duplicates", "moe_permute", "moe_grouped_ffn",
                 "moe_combine"]:
        assert name in syms


def test_library_exports_every_declared_symbol():
    from paper_2506_07366_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2506_07366_amd.build import build
        build(verbose=False)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared_symbols():
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == declared_symbols()
    lib.moe_strerror.restype = ctypes.c_char_p
    assert lib.moe_strerror(0) == b"ok"
    assert lib.moe_strerror(-1) == b"invalid argument"
    assert lib.moe_abi_version() >= 1


def test_host_side_argument_checks_need_no_gpu():
    """Scalar checks fail before anything is enqueued."""
    from paper_2506_07366_amd import binding
    lib = binding.load_library()
    assert lib.moe_route_topk(None, 4, 8, 9, None, None, None) == -1          # k > E
    assert lib.moe_route_topk(None, 4, 2000, 2, None, None, None) == -2       # E above the compile-time limit
    assert lib.moe_route_topk(None, 0, 8, 2, None, None, None) == 0           # empty input is a no-op
    assert lib.moe_histogram(None, -1, 8, None, None) == -1
    assert lib.moe_plan_duplicates(1, None, 8, 2, 3, 2, None, None, None, None, None) == -1   # ceil(E/G) > S
    assert lib.moe_plan_duplicates(7, None, 8, 4, 3, 2, None, None, None, None, None) == -1   # bad mode
    assert lib.moe_combine(None, 1, 4, 100, 2, None, None, None, None) == -2  # row bytes not a multiple of 16
    assert lib.moe_combine(None, 5, 4, 128, 2, None, None, None, None) == -1  # bad dtype
    assert lib.moe_comm_matrix(9, 4, 2, 2, 2, None, None, None, None, None, None, None) == -1   # bad mode
    assert lib.moe_comm_matrix(0, 4, 2, 300, 2, None, None, None, None, None, None, None) == -2  # G above the limit
    assert lib.moe_comm_matrix(0, 4, 2, 2, 2, None, None, None, None, None, None, None) == -1   # no output tables
    assert lib.moe_predictor_update(None, 8, None, None) == -1                  # no buffers
    assert lib.moe_predictor_predict(None, 2000, 10, None, None) == -2          # E above the limit
    assert lib.moe_predictor_predict(None, 8, -1, None, None) == -1             # negative batch size
    assert lib.moe_permute_workspace_bytes(4096, 8, 2, 8, 2) > 0
    assert lib.moe_grouped_ffn_workspace_bytes(8192, 4096, 14336, 16, 1) >= 8192 * 14336 * 2


def test_missing_library_fails_loudly(tmp_path):
    from paper_2506_07366_amd import binding
    with pytest.raises(binding.MoeGpsError):
        binding.load_library(str(tmp_path / "nope.so"))


def test_ffn_workspace_size_rule():
    """Host logic of the FFN workspace: the fp32 slabs of the split tiles are part of it
    exactly when the rule says so (bf16, at most eight rounds of tiles per workgroup, segments
    that are not slivers, at least 16 k-tiles), and the option turns them off and on."""
    from paper_2506_07366_amd import binding
    lib = binding.load_library()
    ws = lib.moe_grouped_ffn_workspace_bytes
    opt = lib.moe_grouped_ffn_set_option
    SPLIT = binding.FFN_OPT_SPLIT_K
    try:
        h_mixtral = 8192 * 14336 * 2
        assert opt(SPLIT, 0) == 0
        base = ws(8192, 4096, 14336, 16, 1)
        assert h_mixtral <= base < h_mixtral + (2 << 20)
        assert opt(SPLIT, -1) == 0
        # Mixtral-shaped batch: 2-3 rounds of tiles.  Room for 5/8 of a round of tiles in half-tile M-tiles (22), 4 parts each
        assert ws(8192, 4096, 14336, 16, 1) - base >= 22 * 4 * 256 * 4096 * 4
        big_auto = ws(262144, 4096, 1536, 160, 1)
        dec_auto = ws(1024, 4096, 1536, 160, 1)
        f32_auto = ws(8192, 4096, 14336, 16, 0)
        assert opt(SPLIT, 0) == 0
        assert ws(262144, 4096, 1536, 160, 1) == big_auto             # many rounds per workgroup: never split
        assert ws(1024, 4096, 1536, 160, 1) == dec_auto               # a few rows per segment: never split
        assert ws(8192, 4096, 14336, 16, 0) == f32_auto               # fp32 path: never split
        assert opt(SPLIT, 1) == 0
        assert ws(1024, 512, 1024, 12, 1) > ws(1024, 512, 64, 12, 1)  # forced, but not with a single k-tile
        assert ws(-1, 64, 64, 1, 1) == 0 and ws(16, 64, 64, 0, 1) == 0
        assert opt(SPLIT, 2) == -1 and opt(99, 0) == -1 and opt(binding.FFN_OPT_TILE1, 3) == -1
    finally:
        opt(SPLIT, -1)
