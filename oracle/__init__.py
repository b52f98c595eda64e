"""ctypes front-end of the CPU oracle (oracle/moe_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
bench's cpu_baseline leg, never by the product package.  It imports nothing
from the HIP path.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math, OpenMP for the row loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


@dataclass
class LayerResult:
    logits: np.ndarray      # [T,E] f64
    topk_idx: np.ndarray    # [T,k] i32
    gate: np.ndarray        # [T,k] f64
    hist: np.ndarray        # [E] i32
    slot_idx: np.ndarray    # [T,k] i32
    miss_list: np.ndarray   # [miss_count] i32
    miss_count: int
    y: np.ndarray           # [T,H] f64


class Oracle:
    """The oracle's entry points bound to one shared library (the default
    instance uses oracle/libmoe_oracle.so; tests that plant mistakes load a
    mutated build through the same class)."""

    def __init__(self, path: Optional[str] = None):
        self._lib = ctypes.CDLL(path or build())
        self._lib.oracle_max_threads.restype = ctypes.c_int

    def max_threads(self) -> int:
        return int(self._lib.oracle_max_threads())

    def set_threads(self, n: int) -> None:
        self._lib.oracle_set_threads(ctypes.c_int(n))

    def router_logits(self, hidden, router_w, bias=None) -> np.ndarray:
        hidden = _c(hidden, np.uint16)
        router_w = _c(router_w, np.float32)
        bias = _c(bias, np.float32)
        T, H = hidden.shape
        E = router_w.shape[0]
        assert router_w.shape == (E, H)
        out = np.empty((T, E), dtype=np.float64)
        self._lib.oracle_router_logits(_p(hidden), _p(router_w), _p(bias), T, H, E, _p(out))
        return out

    def topk_gate(self, logits, k: int):
        logits = _c(logits, np.float64)
        T, E = logits.shape
        assert 1 <= k <= E
        idx = np.empty((T, k), dtype=np.int32)
        gate = np.empty((T, k), dtype=np.float64)
        self._lib.oracle_topk_gate(_p(logits), T, E, k, _p(idx), _p(gate))
        return idx, gate

    def expert_histogram(self, topk_idx, E: int) -> np.ndarray:
        topk_idx = _c(topk_idx, np.int32)
        T, k = topk_idx.shape
        hist = np.empty(E, dtype=np.int32)
        self._lib.oracle_expert_histogram(_p(topk_idx), T, k, E, _p(hist))
        return hist

    def slot_resolve(self, topk_idx, slot_table):
        topk_idx = _c(topk_idx, np.int32)
        slot_table = _c(slot_table, np.int32)
        T, k = topk_idx.shape
        slot_idx = np.empty((T, k), dtype=np.int32)
        miss = np.empty(T * k, dtype=np.int32)
        cnt = np.zeros(1, dtype=np.int32)
        self._lib.oracle_slot_resolve(_p(topk_idx), _p(slot_table), T, k, _p(slot_idx), _p(miss), _p(cnt))
        n = int(cnt[0])
        return slot_idx, miss[:n].copy(), n

    def routed_ffn(self, hidden, topk_idx, gate, slot_table, w_gate, w_up, w_down) -> np.ndarray:
        hidden = _c(hidden, np.uint16)
        topk_idx = _c(topk_idx, np.int32)
        gate = _c(gate, np.float64)
        slot_table = _c(slot_table, np.int32)
        w_gate, w_up, w_down = _c(w_gate, np.uint16), _c(w_up, np.uint16), _c(w_down, np.uint16)
        T, H = hidden.shape
        E, F, H2 = w_gate.shape
        assert H2 == H and w_up.shape == (E, F, H) and w_down.shape == (E, H, F)
        k = topk_idx.shape[1]
        y = np.empty((T, H), dtype=np.float64)
        self._lib.oracle_routed_ffn(_p(hidden), _p(topk_idx), _p(gate), _p(slot_table), _p(w_gate),
                                    _p(w_up), _p(w_down), T, H, F, k, _p(y))
        return y

    def shared_ffn_add(self, hidden, sh_gate, sh_up, sh_down, y) -> np.ndarray:
        hidden = _c(hidden, np.uint16)
        sh_gate, sh_up, sh_down = _c(sh_gate, np.uint16), _c(sh_up, np.uint16), _c(sh_down, np.uint16)
        T, H = hidden.shape
        n, Fs, _ = sh_gate.shape
        assert sh_up.shape == (n, Fs, H) and sh_down.shape == (n, H, Fs)
        assert y.dtype == np.float64 and y.flags.c_contiguous
        self._lib.oracle_shared_ffn_add(_p(hidden), _p(sh_gate), _p(sh_up), _p(sh_down), T, H, Fs, n, _p(y))
        return y

    def utility_step(self, f, f_prev, s, th_up, th_dn, K: int, lam_num: int, lam_den: int):
        """One step of Alg. 1 for the N experts of one layer; returns the new (f_prev, s, th_up, th_dn)."""
        f = _c(f, np.int32)
        f_prev, s = np.array(f_prev, dtype=np.int32), np.array(s, dtype=np.int32)
        th_up, th_dn = np.array(th_up, dtype=np.int32), np.array(th_dn, dtype=np.int32)
        N = f.shape[0]
        assert f_prev.shape == s.shape == th_up.shape == th_dn.shape == (N,)
        self._lib.oracle_utility_step(_p(f), _p(f_prev), _p(s), _p(th_up), _p(th_dn), N, K, lam_num, lam_den)
        return f_prev, s, th_up, th_dn

    def prefetch_counts(self, s, slot_table, K: int) -> np.ndarray:
        """n(tau), tau = 0..K: experts with utility >= tau that hold no cache slot."""
        s = _c(s, np.int32)
        slot_table = _c(slot_table, np.int32)
        n_tau = np.empty(K + 1, dtype=np.int32)
        self._lib.oracle_prefetch_counts(_p(s), _p(slot_table), s.shape[0], K, _p(n_tau))
        return n_tau

    def balance_threshold(self, f, n_tau, r_c, r_g, K: int, gamma: int, k: int, t_cpu: float, t_gpu: float,
                          t_io: float, t_draft: float, l_target: int, w_expert: int, vram_left: int):
        """tau* of one layer and (b, T_cpu[0..K], T_gpu[0..K]); entry 0 of the time tables is NaN."""
        f, n_tau = _c(f, np.int32), _c(n_tau, np.int32)
        r_c, r_g = _c(r_c, np.float64), _c(r_g, np.float64)
        assert n_tau.shape == r_c.shape == r_g.shape == (K + 1,)
        b = np.zeros(1, dtype=np.int32)
        tc = np.full(K + 1, np.nan)
        tg = np.full(K + 1, np.nan)
        fn = self._lib.oracle_balance_threshold
        fn.restype = ctypes.c_int
        fn.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int] * 4 + [ctypes.c_double] * 4 + [ctypes.c_int,
                       ctypes.c_int64, ctypes.c_int64] + [ctypes.c_void_p] * 3
        tau = fn(_p(f), _p(n_tau), _p(r_c), _p(r_g), f.shape[0], K, gamma, k, t_cpu, t_gpu, t_io, t_draft,
                 l_target, w_expert, vram_left, _p(b), _p(tc), _p(tg))
        return int(tau), int(b[0]), tc, tg

    def cache_plan(self, s, in_use, slot_table, C: int, K: int, tau: int, budget: int):
        """One planning step of the cache manager; returns (new_slot_table, evict_list, fetch_list, fetch_slot)."""
        s, in_use = _c(s, np.int32), _c(in_use, np.int32)
        tab = np.array(slot_table, dtype=np.int32)
        N = s.shape[0]
        ev, fl, fs = (np.full(max(N, 1), -1, dtype=np.int32) for _ in range(3))
        ne, nf = np.zeros(1, dtype=np.int32), np.zeros(1, dtype=np.int32)
        self._lib.oracle_cache_plan(_p(s), _p(in_use), _p(tab), N, C, K, tau, budget, _p(ev), _p(ne), _p(fl), _p(fs),
                                    _p(nf))
        return tab, ev[:int(ne[0])].copy(), fl[:int(nf[0])].copy(), fs[:int(nf[0])].copy()

    def verify_layer(self, hidden, router_w, router_bias, slot_table, w_gate, w_up, w_down, k: int,
                     sh_gate=None, sh_up=None, sh_down=None) -> LayerResult:
        hidden = _c(hidden, np.uint16)
        router_w = _c(router_w, np.float32)
        router_bias = _c(router_bias, np.float32)
        slot_table = _c(slot_table, np.int32)
        w_gate, w_up, w_down = _c(w_gate, np.uint16), _c(w_up, np.uint16), _c(w_down, np.uint16)
        sh_gate, sh_up, sh_down = _c(sh_gate, np.uint16), _c(sh_up, np.uint16), _c(sh_down, np.uint16)
        T, H = hidden.shape
        E, F, _ = w_gate.shape
        assert router_w.shape == (E, H) and slot_table.shape == (E,)
        assert w_up.shape == (E, F, H) and w_down.shape == (E, H, F)
        n_sh, Fs = (0, 0) if sh_gate is None else sh_gate.shape[:2]
        logits = np.empty((T, E), dtype=np.float64)
        idx = np.empty((T, k), dtype=np.int32)
        gate = np.empty((T, k), dtype=np.float64)
        hist = np.empty(E, dtype=np.int32)
        slot_idx = np.empty((T, k), dtype=np.int32)
        miss = np.empty(T * k, dtype=np.int32)
        cnt = np.zeros(1, dtype=np.int32)
        y = np.empty((T, H), dtype=np.float64)
        self._lib.oracle_verify_layer(_p(hidden), _p(router_w), _p(router_bias), _p(slot_table), _p(w_gate),
                                  _p(w_up), _p(w_down), _p(sh_gate), _p(sh_up), _p(sh_down), T, H, E, k, F,
                                  int(n_sh), int(Fs), _p(logits), _p(idx), _p(gate), _p(hist), _p(slot_idx),
                                  _p(miss), _p(cnt), _p(y))
        n = int(cnt[0])
        return LayerResult(logits, idx, gate, hist, slot_idx, miss[:n].copy(), n, y)

    def layer_from_inputs(self, li) -> LayerResult:
        """Run the oracle on a synth.LayerInputs bundle."""
        return self.verify_layer(li.hidden, li.router_w, li.router_bias, li.slot_table, li.w_gate, li.w_up,
                            li.w_down, li.shape.k, li.sh_gate, li.sh_up, li.sh_down)


_default: Optional[Oracle] = None


def default() -> Oracle:
    global _default
    if _default is None:
        _default = Oracle()
    return _default


def __getattr__(name):  # module-level access: oracle.topk_gate(...) -> default().topk_gate(...)
    if name.startswith("_"):
        raise AttributeError(name)
    return getattr(default(), name)
