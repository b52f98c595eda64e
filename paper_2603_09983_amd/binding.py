"""Thin Python binding of libmoe_spac.so: argument marshalling only.

Every function has the name and argument meaning of its C entry point in
include/moe_spac.h.  Tensors are torch CUDA(HIP) tensors used as typed device
pointers; the stream is torch's current stream unless one is given.  There is
no fallback: if the library is not built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# (MOE_SPAC_LIB names another build of the same library, e.g. the one with the timeline stamps)
LIB_PATH = os.environ.get("MOE_SPAC_LIB") or os.path.join(_HERE, "libmoe_spac.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'` "
        "(hipcc, gfx950). There is no CPU or PyTorch fallback for the MoE layer.")

_lib = ctypes.CDLL(LIB_PATH)

OK, ERR_NULL, ERR_SHAPE, ERR_ALIGN, ERR_WORKSPACE, ERR_LAUNCH, ERR_SCRATCH = 0, -1, -2, -3, -4, -5, -6
STATIC_SCRATCH_BYTES = 16 << 20


class MoeShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("T", "H", "E", "k", "F", "C", "n_shared", "F_shared", "launch_form")]


_vp, _sz, _i = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
_lib.moe_status_string.restype = ctypes.c_char_p
_lib.moe_status_string.argtypes = [_i]
_lib.moe_workspace_bytes.argtypes = [ctypes.POINTER(MoeShape), ctypes.POINTER(_sz)]
_lib.moe_workspace_init.argtypes = [_vp, _sz, _vp]
_lib.moe_workspace_status.argtypes = [_vp, _sz, _vp]
_lib.moe_workspace_wait_test.argtypes = [_vp, _sz, ctypes.c_uint, ctypes.c_uint, _vp]
_lib.moe_route_topk.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.moe_expert_histogram.argtypes = [_vp, _i, _i, _i, _vp, _vp]
_lib.moe_slot_resolve.argtypes = [_vp, _vp, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.moe_grouped_ffn.argtypes = [_vp] * 6 + [_i] * 5 + [_vp, _i, _i, _vp, _sz, _vp]
_lib.moe_verify_layer.argtypes = [ctypes.POINTER(MoeShape)] + [_vp] * 17 + [_i, _i, _vp, _sz, _vp]
_lib.moe_verify_layer_static.argtypes = [ctypes.POINTER(MoeShape)] + [_vp] * 17 + [_i, _i, _vp]
_lib.moe_verify_layer_static.restype = _i
class BalanceParams(ctypes.Structure):
    _fields_ = [("t_cpu", ctypes.c_double), ("t_gpu", ctypes.c_double), ("t_io", ctypes.c_double),
                ("t_draft", ctypes.c_double), ("l_target", ctypes.c_int), ("w_expert_bytes", ctypes.c_int64),
                ("vram_left_bytes", ctypes.c_int64)]


_lib.moe_balance_threshold.argtypes = [_vp] * 4 + [_i] * 5 + [ctypes.POINTER(BalanceParams), _vp, _vp, _vp]
_lib.moe_balance_threshold.restype = _i
_lib.moe_cache_plan.argtypes = [_vp] * 5 + [_i] * 4 + [_vp] * 6
_lib.moe_cache_plan.restype = _i
_lib.moe_pool_load.argtypes = [_vp] * 9 + [_i] * 3 + [_vp]
_lib.moe_pool_load.restype = _i
_lib.moe_utility_init.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _vp]
_lib.moe_utility_update.argtypes = [_vp] * 7 + [_i] * 5 + [_vp]
for _f in ("moe_utility_init", "moe_utility_update", "moe_workspace_bytes", "moe_workspace_init", "moe_workspace_status", "moe_workspace_wait_test", "moe_route_topk", "moe_expert_histogram",
           "moe_slot_resolve", "moe_grouped_ffn", "moe_verify_layer"):
    getattr(_lib, _f).restype = _i

_lib.moe_profile_enable.argtypes = [_i]
_lib.moe_profile_enable.restype = _i
_lib.moe_profile_read.argtypes = [_i, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_i)]
_lib.moe_profile_read.restype = _i
_lib.moe_profile_event_overhead.argtypes = [_vp, _i, ctypes.POINTER(ctypes.c_double)]
_lib.moe_profile_event_overhead.restype = _i
_lib.moe_profile_stream_timeline.argtypes = [ctypes.c_void_p, _sz]
_lib.moe_profile_stream_timeline.restype = _i
_lib.moe_profile_kernel_name.argtypes = [_i]
_lib.moe_profile_kernel_name.restype = ctypes.c_char_p
KERNEL_ROUTE, KERNEL_LISTS, KERNEL_FFN, KERNEL_COMBINE, KERNEL_DOWN, KERNEL_ESTIMATOR, KERNEL_BALANCER, KERNEL_CACHE_PLAN, KERNEL_POOL_LOAD, KERNEL_LAYER, KERNEL_KINDS = 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10

EXPORTS = ("moe_profile_stream_timeline", "moe_cache_plan", "moe_pool_load", "moe_balance_threshold", "moe_utility_init", "moe_utility_update", "moe_profile_event_overhead", "moe_profile_enable", "moe_profile_read", "moe_profile_kernel_name", "moe_status_string", "moe_workspace_bytes", "moe_workspace_init", "moe_workspace_status", "moe_workspace_wait_test", "moe_route_topk",
           "moe_expert_histogram", "moe_slot_resolve", "moe_grouped_ffn", "moe_verify_layer", "moe_verify_layer_static")


class MoeError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: status {code}: {moe_status_string(code)}")


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device-resident contiguous tensors only")
    return t.data_ptr()


def _ptr_store(t: torch.Tensor):
    """The expert store of moe_pool_load: device memory, or pinned host memory (which the runtime maps into
    the device under the same address)."""
    if not t.is_contiguous() or not (t.is_cuda or t.is_pinned()):
        raise ValueError("the expert store must be a contiguous tensor in device memory or in pinned host memory")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check(rc: int, where: str, check: bool) -> int:
    if check and rc != OK:
        raise MoeError(rc, where)
    return rc


def moe_status_string(status: int) -> str:
    return _lib.moe_status_string(status).decode()


def moe_profile_enable(on: bool) -> int:
    return _check(_lib.moe_profile_enable(int(on)), "moe_profile_enable", True)


def moe_profile_read(kind: int):
    """(total_ms, launches) of one kernel kind since moe_profile_enable(True); sync first."""
    ms, n = ctypes.c_double(0.0), _i(0)
    _check(_lib.moe_profile_read(kind, ctypes.byref(ms), ctypes.byref(n)), "moe_profile_read", True)
    return float(ms.value), int(n.value)


def moe_profile_stream_timeline():
    """([2, 1024, 8], [1024, 24]) uint64 (numpy): the two streaming kernels' records and the one-launch layer
    kernel's; None when the loaded library is not a tracing build."""
    import numpy as np
    words = np.zeros(2 * 1024 * 8 + 1024 * 24, dtype=np.uint64)
    rc = _lib.moe_profile_stream_timeline(ctypes.c_void_p(words.ctypes.data), words.size)
    if rc == ERR_SHAPE:
        return None
    _check(rc, "moe_profile_stream_timeline", True)
    return words[:2 * 1024 * 8].reshape(2, 1024, 8), words[2 * 1024 * 8:].reshape(1024, 24)


def moe_profile_event_overhead(pairs: int = 256, stream=None) -> float:
    """Mean interval (ms) of an event pair with nothing between its two records."""
    ms = ctypes.c_double(0.0)
    _check(_lib.moe_profile_event_overhead(_stream(stream), pairs, ctypes.byref(ms)), "moe_profile_event_overhead", True)
    return float(ms.value)


def moe_profile_kernel_name(kind: int) -> str:
    return _lib.moe_profile_kernel_name(kind).decode()


LAUNCH_AUTO, LAUNCH_THREE, LAUNCH_TWO, LAUNCH_ONE, LAUNCH_ROUTE_PLUS_ONE = 0, 1, 2, 3, 4


def make_shape(T, H, E, k, F, C, n_shared=0, F_shared=0, launch_form=LAUNCH_AUTO) -> MoeShape:
    return MoeShape(T, H, E, k, F, C, n_shared, F_shared, launch_form)


def with_form(shape: MoeShape, launch_form: int) -> MoeShape:
    return MoeShape(shape.T, shape.H, shape.E, shape.k, shape.F, shape.C, shape.n_shared, shape.F_shared, launch_form)


def moe_workspace_bytes(shape: MoeShape) -> int:
    out = _sz(0)
    rc = _lib.moe_workspace_bytes(ctypes.byref(shape), ctypes.byref(out))
    _check(rc, "moe_workspace_bytes", True)
    return int(out.value)


def moe_workspace_init(workspace: torch.Tensor, stream=None, check=True) -> int:
    return _check(_lib.moe_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                          _stream(stream)), "moe_workspace_init", check)


def moe_workspace_status(workspace: torch.Tensor, stream=None, check=True) -> int:
    return _check(_lib.moe_workspace_status(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                            _stream(stream)), "moe_workspace_status", check)


def moe_workspace_wait_test(workspace: torch.Tensor, poll_limit: int, stamp_skew: int, stream=None, check=True) -> int:
    return _check(_lib.moe_workspace_wait_test(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                               poll_limit, stamp_skew, _stream(stream)), "moe_workspace_wait_test", check)


def new_workspace(shape: MoeShape, device="cuda") -> torch.Tensor:
    """Device buffer of moe_workspace_bytes(shape) bytes with a cleared control block."""
    ws = torch.empty(moe_workspace_bytes(shape), dtype=torch.uint8, device=device)
    moe_workspace_init(ws)
    return ws


def moe_route_topk(hidden, router_w, router_bias, T, H, E, k, topk_idx, topk_w, logits_opt, workspace,
                   stream=None, check=True) -> int:
    rc = _lib.moe_route_topk(_ptr(hidden), _ptr(router_w), _ptr(router_bias), T, H, E, k, _ptr(topk_idx),
                             _ptr(topk_w), _ptr(logits_opt), _ptr(workspace),
                             0 if workspace is None else workspace.numel(), _stream(stream))
    return _check(rc, "moe_route_topk", check)


def moe_expert_histogram(topk_idx, T, k, E, hist, stream=None, check=True) -> int:
    return _check(_lib.moe_expert_histogram(_ptr(topk_idx), T, k, E, _ptr(hist), _stream(stream)),
                  "moe_expert_histogram", check)


def moe_slot_resolve(topk_idx, slot_table, T, k, E, C, slot_idx, miss_list, miss_count, workspace,
                     stream=None, check=True) -> int:
    rc = _lib.moe_slot_resolve(_ptr(topk_idx), _ptr(slot_table), T, k, E, C, _ptr(slot_idx), _ptr(miss_list),
                               _ptr(miss_count), _ptr(workspace),
                               0 if workspace is None else workspace.numel(), _stream(stream))
    return _check(rc, "moe_slot_resolve", check)


def moe_grouped_ffn(hidden, topk_w, slot_idx, w_gate, w_up, w_down, T, H, F, k, C, out, out_bf16, accumulate,
                    workspace, stream=None, check=True) -> int:
    rc = _lib.moe_grouped_ffn(_ptr(hidden), _ptr(topk_w), _ptr(slot_idx), _ptr(w_gate), _ptr(w_up),
                              _ptr(w_down), T, H, F, k, C, _ptr(out), int(out_bf16), int(accumulate),
                              _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream))
    return _check(rc, "moe_grouped_ffn", check)


def moe_verify_layer(shape: MoeShape, hidden, router_w, router_bias, slot_table, w_gate, w_up, w_down,
                     shared_gate, shared_up, shared_down, topk_idx, topk_w, hist, slot_idx, miss_list,
                     miss_count, out, out_bf16, accumulate, workspace, stream=None, check=True) -> int:
    rc = _lib.moe_verify_layer(ctypes.byref(shape), _ptr(hidden), _ptr(router_w), _ptr(router_bias),
                               _ptr(slot_table), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(shared_gate),
                               _ptr(shared_up), _ptr(shared_down), _ptr(topk_idx), _ptr(topk_w), _ptr(hist),
                               _ptr(slot_idx), _ptr(miss_list), _ptr(miss_count), _ptr(out), int(out_bf16),
                               int(accumulate), _ptr(workspace), 0 if workspace is None else workspace.numel(),
                               _stream(stream))
    return _check(rc, "moe_verify_layer", check)


def moe_verify_layer_static(shape: MoeShape, hidden, router_w, router_bias, slot_table, w_gate, w_up, w_down,
                            shared_gate, shared_up, shared_down, topk_idx, topk_w, hist, slot_idx, miss_list,
                            miss_count, out, out_bf16, accumulate, stream=None, check=True) -> int:
    rc = _lib.moe_verify_layer_static(ctypes.byref(shape), _ptr(hidden), _ptr(router_w), _ptr(router_bias),
                                      _ptr(slot_table), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(shared_gate),
                                      _ptr(shared_up), _ptr(shared_down), _ptr(topk_idx), _ptr(topk_w), _ptr(hist),
                                      _ptr(slot_idx), _ptr(miss_list), _ptr(miss_count), _ptr(out), int(out_bf16),
                                      int(accumulate), _stream(stream))
    return _check(rc, "moe_verify_layer_static", check)


def moe_utility_init(f_prev, s, theta_up, theta_dn, L, N, gamma, stream=None, check=True) -> int:
    return _check(_lib.moe_utility_init(_ptr(f_prev), _ptr(s), _ptr(theta_up), _ptr(theta_dn), L, N, gamma,
                                        _stream(stream)), "moe_utility_init", check)


def moe_utility_update(f, f_prev, s, theta_up, theta_dn, slot_table, n_tau, L, N, K, lam_num, lam_den,
                       stream=None, check=True) -> int:
    rc = _lib.moe_utility_update(_ptr(f), _ptr(f_prev), _ptr(s), _ptr(theta_up), _ptr(theta_dn),
                                 _ptr(slot_table), _ptr(n_tau), L, N, K, lam_num, lam_den, _stream(stream))
    return _check(rc, "moe_utility_update", check)


def moe_balance_threshold(f, n_tau, r_c, r_g, L, N, K, gamma, k, params: BalanceParams, tau_out, b_out=None,
                          stream=None, check=True) -> int:
    rc = _lib.moe_balance_threshold(_ptr(f), _ptr(n_tau), _ptr(r_c), _ptr(r_g), L, N, K, gamma, k,
                                    ctypes.byref(params), _ptr(tau_out), _ptr(b_out), _stream(stream))
    return _check(rc, "moe_balance_threshold", check)


def moe_cache_plan(s, in_use, slot_table, tau, budget, L, N, C, K, evict_list, n_evict, fetch_list, fetch_slot,
                   n_fetch, stream=None, check=True) -> int:
    rc = _lib.moe_cache_plan(_ptr(s), _ptr(in_use), _ptr(slot_table), _ptr(tau), _ptr(budget), L, N, C, K,
                             _ptr(evict_list), _ptr(n_evict), _ptr(fetch_list), _ptr(fetch_slot), _ptr(n_fetch),
                             _stream(stream))
    return _check(rc, "moe_cache_plan", check)


def moe_pool_load(store_gate, store_up, store_down, pool_gate, pool_up, pool_down, fetch_list, fetch_slot, n_fetch,
                  max_fetch, H, F, stream=None, check=True) -> int:
    rc = _lib.moe_pool_load(_ptr_store(store_gate), _ptr_store(store_up), _ptr_store(store_down), _ptr(pool_gate), _ptr(pool_up),
                            _ptr(pool_down), _ptr(fetch_list), _ptr(fetch_slot), _ptr(n_fetch), max_fetch, H, F,
                            _stream(stream))
    return _check(rc, "moe_pool_load", check)


# ---------------------------------------------------------------------------
# Convenience holder: device buffers for one layer (allocation and marshalling
# only; every step of the layer runs in the library's kernels).
# ---------------------------------------------------------------------------
@dataclass
class LayerBuffers:
    shape: MoeShape
    topk_idx: torch.Tensor
    topk_w: torch.Tensor
    hist: torch.Tensor
    slot_idx: torch.Tensor
    miss_list: torch.Tensor
    miss_count: torch.Tensor
    out: torch.Tensor
    workspace: torch.Tensor

    @staticmethod
    def allocate(shape: MoeShape, out_bf16: bool = False, device="cuda") -> "LayerBuffers":
        T, k, E, H = shape.T, shape.k, shape.E, shape.H
        i32 = dict(dtype=torch.int32, device=device)
        return LayerBuffers(
            shape,
            torch.empty((T, k), **i32), torch.empty((T, k), dtype=torch.float32, device=device),
            torch.empty(E, **i32), torch.empty((T, k), **i32), torch.empty(T * k, **i32),
            torch.empty(1, **i32),
            torch.empty((T, H), dtype=torch.bfloat16 if out_bf16 else torch.float32, device=device),
            new_workspace(shape, device))
