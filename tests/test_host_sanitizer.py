"""Host side of the library under the undefined-behaviour sanitizer (no GPU needed).

The library is compiled once more with `-fsanitize=undefined -fsanitize-trap=undefined` on the
host pass only (the device pass is untouched) and a child process calls every size query and the
argument checks of every entry point with extreme, zero and negative values.  Undefined behaviour
in the host arithmetic (a signed overflow in a size computation, a bad shift) ends the child
with a trap; a wrong answer to an invalid argument fails the assertion in the child.
"""
import os
import shutil
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2506_07366_amd", "csrc")
SOURCES = ["api", "route_topk", "histogram", "plan", "permute", "grouped_ffn", "combine", "comm", "predictor"]


def _hipcc():
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    return None


@pytest.fixture(scope="module")
def sanitized_library(tmp_path_factory):
    hipcc = _hipcc()
    if hipcc is None:
        pytest.skip("hipcc not found")
    out = tmp_path_factory.mktemp("ubsan")
    flags = ["--offload-arch=gfx950", "-O1", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fsanitize-trap=undefined", "-I", os.path.join(ROOT, "include")]
    procs = []
    for s in SOURCES:
        obj = str(out / (s + ".o"))
        procs.append((s, obj, subprocess.Popen([hipcc, *flags, "-c", os.path.join(CSRC, s + ".hip"), "-o", obj],
                                               stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)))
    objs = []
    for s, obj, p in procs:
        _, err = p.communicate()
        assert p.returncode == 0, f"{s}: {err}"
        objs.append(obj)
    lib = str(out / "libmoegps_ubsan.so")
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", lib], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return lib


CHILD = textwrap.dedent('''
    import ctypes, itertools, sys
    lib = ctypes.CDLL(sys.argv[1])
    c_int, c_i64, c_sz, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_size_t, ctypes.c_void_p
    I32 = [0, 1, -1, 2, 7, 64, 4096, 65536, 2**20, 2**24 + 1, 2**31 - 1, -2**31]
    I64 = I32 + [2**31, 2**40, 2**62, 2**63 - 1, -2**63]
    n = 0

    def sweep(fn, argtypes, pools, restype=c_sz):
        global n
        fn.argtypes, fn.restype = argtypes, restype
        for args in itertools.product(*pools):
            fn(*args)
            n += 1

    D = [0, 1, 2]
    sweep(lib.moe_grouped_ffn_workspace_bytes, [c_i64, c_int, c_int, c_int, c_int], [I64, I32, I32, I32, D])
    sweep(lib.moe_permute_workspace_bytes, [c_int] * 5, [I32, I32, [1, 16, 17, -1, 2**31 - 1], I32, [1, 16, 2**31 - 1]])
    sweep(lib.moe_packed_weights_bytes, [c_int] * 4, [I32, I32, I32, D])
    sweep(lib.moe_packed_weights_relu_bytes, [c_int] * 4, [I32, I32, I32, D])
    print("size queries", n, flush=True)

    # sane answers where the arguments are sane, zero where they are not
    f = lib.moe_grouped_ffn_workspace_bytes
    assert f(8192, 4096, 14336, 16, 1) >= 8192 * 14336 * 2
    assert f(-1, 64, 64, 1, 1) == 0 and f(2**31, 64, 64, 1, 1) == 0 and f(16, 64, 64, 0, 1) == 0
    assert lib.moe_permute_workspace_bytes(4096, 8, 2, 8, 2) > 0
    assert lib.moe_permute_workspace_bytes(-1, 8, 2, 8, 2) == 0

    # every entry point refuses invalid shapes before it touches a pointer or the GPU
    OK, INVALID, UNSUPPORTED = 0, -1, -2
    bad = (INVALID, UNSUPPORTED)
    def call(name, argtypes, *args):
        print("call", name, [a for a in args if a is not None], flush=True)
        fn = getattr(lib, name)
        fn.argtypes, fn.restype = argtypes, c_int
        return fn(*args)
    assert call("moe_route_topk", [vp, c_int, c_int, c_int, vp, vp, vp], None, -1, 8, 2, None, None, None) in bad
    assert call("moe_route_topk", [vp, c_int, c_int, c_int, vp, vp, vp], None, 16, 8, 9, None, None, None) in bad
    assert call("moe_route_topk", [vp, c_int, c_int, c_int, vp, vp, vp], None, 16, 2**31 - 1, 2, None, None, None) in bad
    assert call("moe_histogram", [vp, c_i64, c_int, vp, vp], None, -1, 8, None, None) in bad
    assert call("moe_histogram", [vp, c_i64, c_int, vp, vp], None, 16, 0, None, None) in bad
    assert call("moe_plan_duplicates", [c_int, vp, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp],
                1, None, 8, 2**31 - 1, 2**31 - 1, 1, None, None, None, None, None) in bad
    assert call("moe_plan_duplicates", [c_int, vp, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp],
                7, None, 8, 8, 2, 1, None, None, None, None, None) in bad
    assert call("moe_plan_duplicates", [c_int, vp, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp],
                1, None, 64, 4, 2, 1, None, None, None, None, None) in bad     # 16 homes do not fit 2 slots
    perm_t = [c_int, vp, c_int, c_int, c_int, c_int, c_int, c_int, c_int] + [vp] * 12 + [c_sz, vp]
    for T, d, E, k, G, S in [(-1, 64, 8, 2, 8, 2), (16, 64, 8, 9, 8, 2), (16, 64, 2**31 - 1, 2, 8, 2),
                             (16, 64, 8, 2, 2**31 - 1, 2**31 - 1), (2**31 - 1, 64, 8, 16, 8, 2), (16, 63, 8, 2, 8, 2)]:
        assert call("moe_permute", perm_t, 1, None, 1, T, d, E, k, G, S, *([None] * 12), 0, None) != OK
    static_t = perm_t[:9] + [vp] * 11 + [vp]
    assert call("moe_permute_static", static_t, 1, None, 1, -1, 64, 8, 2, 8, 2, *([None] * 11), None) != OK
    assert call("moe_permute_static", static_t, 1, None, 1, 2**31 - 1, 64, 1024, 16, 256, 8, *([None] * 11), None) != OK
    comm_t = [c_int] * 5 + [vp] * 7
    assert call("moe_comm_matrix", comm_t, 1, -1, 2, 8, 2, *([None] * 7)) != OK
    assert call("moe_comm_matrix", comm_t, 1, 2**31 - 1, 16, 2**31 - 1, 2**31 - 1, *([None] * 7)) != OK
    assert call("moe_predictor_update", [vp, c_int, vp, vp], None, 0, None, None) != OK
    assert call("moe_predictor_predict", [vp, c_int, c_i64, vp, vp], None, 8, -1, None, None) != OK
    assert call("moe_predictor_predict", [vp, c_int, c_i64, vp, vp], None, 8, 2**31, None, None) != OK
    assert call("moe_predictor_predict", [vp, c_int, c_i64, vp, vp], None, 2**31 - 1, 16, None, None) != OK
    ffn_t = [vp, c_int, c_i64, c_int, c_int, c_int, vp, vp, c_int, c_int, c_int, vp, vp, vp, c_sz, vp]
    for A, d, ffn, E, nseg, b, e in [(-1, 64, 64, 8, 16, 0, 16), (2**62, 4096, 14336, 8, 16, 0, 16), (16, 63, 64, 8, 16, 0, 16),
                                     (16, 64, 64, 0, 16, 0, 16), (16, 64, 64, 8, 16, 5, 3), (16, 64, 64, 8, 16, 0, 17),
                                     (2**31 - 1, 2**31 - 64, 2**31 - 1, 8, 2**31 - 1, 0, 2**31 - 1)]:
        for name in ("moe_grouped_ffn", "moe_grouped_ffn_relu"):
            assert call(name, ffn_t, None, 1, A, d, ffn, E, None, None, nseg, b, e, None, None, None, 0, None) != OK
    fused_t = [vp, c_int, c_int, c_int, vp, vp, c_int, c_int, c_int, vp, vp, c_int, c_int, c_int, vp, vp, vp, c_sz, vp]
    assert call("moe_grouped_ffn_fused", fused_t, None, 1, -1, 2, None, None, 64, 64, 8, None, None, 16, 0, 16, None, None, None, 0, None) != OK
    assert call("moe_grouped_ffn_fused", fused_t, None, 1, 2**31 - 1, 16, None, None, 2**31 - 64, 2**31 - 1, 8, None, None, 16, 0, 16, None, None, None, 0, None) != OK
    assert call("moe_combine", [vp, c_int, c_int, c_int, c_int, vp, vp, vp, vp], None, 1, -1, 64, 2, None, None, None, None) != OK
    assert call("moe_combine", [vp, c_int, c_int, c_int, c_int, vp, vp, vp, vp], None, 1, 16, 2**31 - 1, 2**31 - 1, None, None, None, None) != OK
    assert call("moe_grouped_ffn_set_option", [c_int, c_int], 99, 0) != OK
    for code in range(-8, 3):
        lib.moe_strerror.restype = ctypes.c_char_p
        lib.moe_strerror.argtypes = [c_int]
        assert lib.moe_strerror(code)
    print("argument checks ok", flush=True)
''')


def test_host_arithmetic_is_free_of_undefined_behaviour(sanitized_library, tmp_path):
    script = tmp_path / "child.py"
    script.write_text(CHILD)
    r = subprocess.run([sys.executable, str(script), sanitized_library], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, f"child ended with {r.returncode} (a negative code is a signal: the sanitizer's trap)\n{r.stdout[-1500:]}\n{r.stderr[-2000:]}"
    assert "argument checks ok" in r.stdout
