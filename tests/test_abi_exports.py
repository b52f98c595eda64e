"""Host-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2603_09983_amd", "libmoe_spac.so")
HEADER = os.path.join(ROOT, "include", "moe_spac.h")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} not built (run __graft_entry__.build())")
    return ctypes.CDLL(LIB)


def test_header_symbols_are_exported(lib):
    syms = declared_symbols()
    assert {"moe_route_topk", "moe_expert_histogram", "moe_slot_resolve", "moe_grouped_ffn",
            "moe_verify_layer", "moe_workspace_bytes", "moe_workspace_init", "moe_workspace_status",
            "moe_status_string"} <= set(syms)
    for s in syms:
        assert hasattr(lib, s), s


class Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("T", "H", "E", "k", "F", "C", "n_shared", "F_shared", "launch_form")]


def test_workspace_bytes_and_status_strings(lib):
    lib.moe_status_string.restype = ctypes.c_char_p
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert lib.moe_status_string(code)
    n = ctypes.c_size_t(0)
    sh = Shape(9, 2048, 64, 6, 1408, 32, 2, 1408)
    assert lib.moe_workspace_bytes(ctypes.byref(sh), ctypes.byref(n)) == 0
    # at least the activations and per-assignment outputs: A*F*2 + A*H*4 (+ the shared experts' rows)
    assert n.value >= 54 * 1408 * 2 + 54 * 2048 * 4 + 2 * 9 * (1408 * 2 + 2048 * 4)
    big = Shape(128, 2048, 64, 6, 1408, 48, 0, 0)      # large batch, narrow matrices: same layout
    assert lib.moe_workspace_bytes(ctypes.byref(big), ctypes.byref(n)) == 0
    assert n.value >= 768 * 1408 * 2 + 768 * 2048 * 4
    wide = Shape(64, 4096, 8, 2, 14336, 8, 0, 0)       # large batch, wide matrices: per-slice partial sums
    assert lib.moe_workspace_bytes(ctypes.byref(wide), ctypes.byref(n)) == 0
    assert n.value >= 112 * 128 * 4096 * 4
    long_lists = Shape(4096, 128, 16, 8, 128, 16, 0, 0)  # more assignments than the streaming kernels list in LDS
    assert lib.moe_workspace_bytes(ctypes.byref(long_lists), ctypes.byref(n)) == 0
    assert 32768 * 128 * 4 <= n.value < 32768 * 128 * 8  # per-slice partial sums, not the 8-byte entries
    assert lib.moe_workspace_bytes(None, ctypes.byref(n)) == -1
    bad = Shape(9, 2048, 64, 65, 1408, 32, 0, 0)       # k > E
    assert lib.moe_workspace_bytes(ctypes.byref(bad), ctypes.byref(n)) == -2


def test_bad_arguments_are_rejected_before_any_launch(lib):
    vp = ctypes.c_void_p
    lib.moe_route_topk.argtypes = [vp, vp, vp] + [ctypes.c_int] * 4 + [vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.moe_grouped_ffn.argtypes = [vp] * 6 + [ctypes.c_int] * 5 + [vp, ctypes.c_int, ctypes.c_int, vp,
                                                                    ctypes.c_size_t, vp]
    lib.moe_expert_histogram.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
    p = 0x1000  # never dereferenced: every call below must fail its host-side checks first
    assert lib.moe_route_topk(None, p, None, 4, 64, 8, 2, p, p, None, p, 1 << 20, None) == -1
    assert lib.moe_route_topk(p, p, None, 4, 64, 8, 9, p, p, None, p, 1 << 20, None) == -2     # k > E
    assert lib.moe_route_topk(p, p, None, 4, 60, 8, 2, p, p, None, p, 1 << 20, None) == -3     # H % 8
    assert lib.moe_route_topk(p, p, None, 4, 64, 8, 2, p, p, None, p, 16, None) == -4          # workspace
    assert lib.moe_route_topk(p + 4, p, None, 4, 64, 8, 2, p, p, None, p, 1 << 20, None) == -3  # alignment
    assert lib.moe_expert_histogram(None, 4, 2, 8, p, None) == -1
    assert lib.moe_expert_histogram(p, 0, 2, 8, p, None) == -2
    assert lib.moe_grouped_ffn(p, p, p, p, p, p, 4, 76, 64, 2, 4, p, 0, 0, p, 1 << 30, None) == -3   # H % 8
    assert lib.moe_grouped_ffn(p, p, p, p, p, p, 4, 64, 68, 2, 4, p, 0, 0, p, 1 << 30, None) == -3   # F % 8
    assert lib.moe_grouped_ffn(p, p, p, p, p, p, 4, 64, 64, 2, 4, p, 0, 0, p, 64, None) == -4
    # 40 tokens are beyond the streaming kernels' panels, and the other kernel's LDS does not hold rows this wide
    assert lib.moe_grouped_ffn(p, p, p, p, p, p, 40, 8192, 64, 2, 4, p, 0, 0, p, 1 << 30, None) == -2
    assert lib.moe_grouped_ffn(p, p, p, None, p, p, 4, 64, 64, 2, 4, p, 0, 0, p, 1 << 30, None) == -1


def test_timeline_entry_point_of_the_product_build(lib):
    """The product library carries no timeline stamps: the entry point says so and writes nothing."""
    lib.moe_profile_stream_timeline.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
    words = (ctypes.c_ulonglong * (2 * 1024 * 8 + 1024 * 24))()
    words[0] = 7
    assert lib.moe_profile_stream_timeline(None, 2 * 1024 * 8 + 1024 * 24) == -1
    assert lib.moe_profile_stream_timeline(words, 5) == -2
    assert lib.moe_profile_stream_timeline(words, 2 * 1024 * 8 + 1024 * 24) == -2
    assert words[0] == 7


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits without touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
