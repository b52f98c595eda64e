"""Parity of the cache-manager kernels (Sec. 3.4) with the CPU oracle: the planning step bit-exact
(lists, counts, new slot table) over random and edge states, and the whole between-steps chain:
plan -> load the fetched experts into the pools -> the next verify step with the new slot table
gives the oracle's layer for that table."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_09983_amd import synth

pytestmark = pytest.mark.gpu


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _random_state(rng, L, N, C, K, frozen_p=0.2):
    s = rng.integers(0, K + 1, size=(L, N)).astype(np.int32)
    tab = np.full((L, N), -1, dtype=np.int32)
    for l in range(L):
        res = rng.permutation(N)[:int(rng.integers(0, min(N, C) + 1))]
        tab[l, res] = rng.permutation(C)[:len(res)]
    in_use = ((rng.random((L, N)) < frozen_p) & (tab >= 0)).astype(np.int32)
    tau = rng.integers(0, K + 2, size=L).astype(np.int32)
    budget = rng.integers(0, N + 1, size=L).astype(np.int32)
    return s, in_use, tab, tau, budget


def _plan(B, s, in_use, tab, tau, budget, C, K):
    L, N = s.shape
    i32 = dict(dtype=torch.int32, device="cuda")
    d_tab = _dev(tab)
    ev, fl, fs = torch.full((L, N), -9, **i32), torch.full((L, max(C, 1)), -9, **i32), torch.full((L, max(C, 1)), -9, **i32)
    ne, nf = torch.full((L,), -9, **i32), torch.full((L,), -9, **i32)
    B.moe_cache_plan(_dev(s), None if in_use is None else _dev(in_use), d_tab, _dev(tau),
                     None if budget is None else _dev(budget), L, N, C, K, ev, ne, fl, fs, nf)
    torch.cuda.synchronize()
    return d_tab.cpu().numpy(), ev.cpu().numpy(), ne.cpu().numpy(), fl.cpu().numpy(), fs.cpu().numpy(), nf.cpu().numpy()


@pytest.mark.parametrize("L,N,C,K", [(24, 64, 32, 4), (3, 8, 4, 4), (5, 130, 40, 7), (2, 512, 1024, 64), (4, 60, 0, 3),
                                     (6, 64, 64, 1), (1, 1, 1, 1)])
def test_plan_parity(L, N, C, K):
    from paper_2603_09983_amd import binding as B
    rng = np.random.default_rng(31 * N + C + K)
    for trial in range(4):
        s, in_use, tab, tau, budget = _random_state(rng, L, N, C, K)
        if trial == 1:
            budget = None
        if trial == 2:
            in_use = None
        new, ev, ne, fl, fs, nf = _plan(B, s, in_use, tab, tau, budget, C, K)
        for l in range(L):
            o_new, o_ev, o_fl, o_fs = oracle.cache_plan(s[l], np.zeros(N, dtype=np.int32) if in_use is None else in_use[l],
                                                        tab[l], C, K, int(tau[l]), N + C if budget is None else int(budget[l]))
            assert ne[l] == len(o_ev) and nf[l] == len(o_fl), (l, ne[l], len(o_ev), nf[l], len(o_fl))
            assert ev[l, :ne[l]].tolist() == o_ev.tolist()
            assert fl[l, :nf[l]].tolist() == o_fl.tolist() and fs[l, :nf[l]].tolist() == o_fs.tolist()
            assert np.array_equal(new[l], o_new)


def test_plan_errors():
    from paper_2603_09983_amd import binding as B
    i32 = dict(dtype=torch.int32, device="cuda")
    t = torch.zeros((1, 8), **i32)
    one = torch.zeros(1, **i32)
    assert B.moe_cache_plan(t, None, t, one, None, 1, 8, 4, 4, t, one, t, t, one, check=False) == B.OK
    assert B.moe_cache_plan(t, None, t, one, None, 1, 513, 4, 4, t, one, t, t, one, check=False) == B.ERR_SHAPE
    assert B.moe_cache_plan(t, None, t, None, None, 1, 8, 4, 4, t, one, t, t, one, check=False) == B.ERR_NULL
    torch.cuda.synchronize()


def test_plan_load_then_verify_step():
    """Between two verify steps: utilities change, the manager evicts and fetches, the fetched weights
    are copied from the full expert store into the pools, and the next verify step uses the new
    table.  The layer output must be the oracle's for the NEW table (bit-exact routing outputs,
    FFN within tolerance), and the untouched slots must still hold their old experts."""
    from paper_2603_09983_amd import binding as B
    import gpu_util as G
    rec = synth.small_recipe("cache_chain", 77, T=9, H=256, E=64, k=6, F=256, C=24, n_shared=1, F_shared=128)
    li = synth.make_layer(rec)
    d = G.upload(li)
    buf = G.run_layer(d)
    G.check_against_oracle(li, buf, tag="before")
    E, C, K = 64, 24, 4
    rng = np.random.default_rng(9)
    s = rng.integers(0, K + 1, size=(1, E)).astype(np.int32)
    in_use = np.zeros((1, E), dtype=np.int32)
    resident = np.flatnonzero(li.slot_table >= 0)
    in_use[0, resident[:3]] = 1
    tau = np.array([2], dtype=np.int32)
    i32 = dict(dtype=torch.int32, device="cuda")
    d_tab = _dev(li.slot_table.reshape(1, E))
    ev, fl, fs = torch.zeros((1, E), **i32), torch.zeros((1, C), **i32), torch.zeros((1, C), **i32)
    ne, nf = torch.zeros(1, **i32), torch.zeros(1, **i32)
    B.moe_cache_plan(_dev(s), _dev(in_use), d_tab, _dev(tau), None, 1, E, C, K, ev, ne, fl, fs, nf)
    store = [_dev(w.view(np.int16)) for w in (li.w_gate, li.w_up, li.w_down)]   # every expert of the layer, [E,...]
    B.moe_pool_load(*store, d.w_gate, d.w_up, d.w_down, fl[0], fs[0], nf, C, 256, 256)
    torch.cuda.synchronize()
    o_tab, o_ev, o_fl, o_fs = oracle.cache_plan(s[0], in_use[0], li.slot_table, C, K, 2, E + C)
    assert int(nf.item()) == len(o_fl) > 0 and int(ne.item()) == len(o_ev) > 0
    assert np.array_equal(d_tab.cpu().numpy()[0], o_tab)
    # pools: fetched slots hold the fetched experts, kept slots their old ones
    pg = d.w_gate.view(torch.int16).cpu().numpy().view(np.uint16)
    for e in np.flatnonzero(o_tab >= 0):
        assert np.array_equal(pg[o_tab[e]], li.w_gate[e]), e
    # next verify step with the new table
    li.slot_table = o_tab.copy()
    d.slot_table = d_tab[0].contiguous()
    buf = G.run_layer(d, buf)
    G.check_against_oracle(li, buf, tag="after")


def test_full_control_loop_three_steps():
    """verify step -> histogram -> utility update (+ n(tau)) -> threshold -> cache plan -> weight load
    -> next verify step, three times round, every stage against the oracle's own chain."""
    from paper_2603_09983_amd import binding as B
    import gpu_util as G
    E, C, K, gamma, k = 64, 24, 4, 8, 6
    rec = synth.small_recipe("control_loop", 91, T=gamma + 1, H=256, E=E, k=k, F=256, C=C)
    li = synth.make_layer(rec)
    d = G.upload(li)
    store = [_dev(w.view(np.int16)) for w in (li.w_gate, li.w_up, li.w_down)]
    i32 = dict(dtype=torch.int32, device="cuda")
    st = [torch.zeros((1, E), **i32) for _ in range(4)]
    B.moe_utility_init(*st, 1, E, gamma)
    z, th = np.zeros(E, dtype=np.int32), np.full(E, gamma // 2, dtype=np.int32)
    o_st = (z.copy(), z.copy(), th.copy(), th.copy())
    d_tab = _dev(li.slot_table.reshape(1, E))
    d_n, d_tau = torch.zeros((1, K + 1), **i32), torch.zeros(1, **i32)
    ev, fl, fs = torch.zeros((1, E), **i32), torch.zeros((1, C), **i32), torch.zeros((1, C), **i32)
    ne, nf = torch.zeros(1, **i32), torch.zeros(1, **i32)
    rng = np.random.default_rng(4)
    r_c = np.sort(rng.random((1, K + 1)), axis=1)
    r_g = np.ascontiguousarray(np.sort(rng.random((1, K + 1)), axis=1)[:, ::-1])
    p = dict(t_cpu=40.0, t_gpu=3.0, t_io=2.0, t_draft=600.0, l_target=24, w_expert=6 * 256 * 256, vram_left=12 * 6 * 256 * 256)
    params = B.BalanceParams(p["t_cpu"], p["t_gpu"], p["t_io"], p["t_draft"], p["l_target"], p["w_expert"], p["vram_left"])
    o_tab = li.slot_table.copy()
    buf = None
    moved = 0
    for step in range(3):
        li_t = synth.make_layer(rec, hidden_seed=500 + step)
        li_t.slot_table = o_tab.copy()
        d.hidden = G.upload(li_t).hidden
        d.slot_table = d_tab[0].contiguous()
        buf = G.run_layer(d, buf)
        G.check_against_oracle(li_t, buf, tag=f"step{step}")
        hist = buf.hist.view(1, E)
        B.moe_utility_update(hist, *st, d_tab, d_n, 1, E, K, 1, 2)
        B.moe_balance_threshold(hist, d_n, _dev(r_c), _dev(r_g), 1, E, K, gamma, k, params, d_tau)
        B.moe_cache_plan(st[1], None, d_tab, d_tau, None, 1, E, C, K, ev, ne, fl, fs, nf)
        B.moe_pool_load(*store, d.w_gate, d.w_up, d.w_down, fl[0], fs[0], nf, C, 256, 256)
        torch.cuda.synchronize()
        ref = oracle.layer_from_inputs(li_t)
        o_st = oracle.utility_step(ref.hist, *o_st, K, 1, 2)
        n_tau = oracle.prefetch_counts(o_st[1], o_tab, K)
        tau = oracle.balance_threshold(ref.hist, n_tau, r_c[0], r_g[0], K, gamma, k, **p)[0]
        o_tab, o_ev, o_fl, o_fs = oracle.cache_plan(o_st[1], np.zeros(E, dtype=np.int32), o_tab, C, K, tau, E + C)
        assert int(d_tau.item()) == tau, step
        assert np.array_equal(st[1].cpu().numpy()[0], o_st[1])
        assert np.array_equal(d_tab.cpu().numpy()[0], o_tab), step
        assert fl[0, :len(o_fl)].cpu().tolist() == o_fl.tolist() and int(nf.item()) == len(o_fl)
        moved += len(o_fl) + len(o_ev)
    assert moved > 0   # the loop did move experts


@pytest.mark.parametrize("gen,steps", [("sampled", 120), ("smooth", 120)])
def test_closed_loop_long_trace(gen, steps):
    """24 layers through 120 inference steps of the closed loop, the device's slot tables feeding its own
    next step: frequencies -> utility update + n(tau) -> threshold -> cache plan (frozen flags, fetch
    budget).  Utilities, boundaries, n(tau), tau, lists and tables bit-exact against the oracle's chain at
    every step."""
    from paper_2603_09983_amd import binding as B
    import traces
    L, N, C, K, gamma, k = 24, 64, 32, 4, 8, 6
    rng = np.random.default_rng(77)
    make = traces.sampled_trace if gen == "sampled" else traces.smooth_trace
    f = make(rng, L, N, gamma + 1, k, steps, 0.1, 40)
    i32 = dict(dtype=torch.int32, device="cuda")
    st = [torch.zeros((L, N), **i32) for _ in range(4)]
    B.moe_utility_init(*st, L, N, gamma)
    tab0 = np.full((L, N), -1, dtype=np.int32)
    for l in range(L):
        tab0[l, rng.permutation(N)[:C]] = rng.permutation(C)
    d_tab = _dev(tab0)
    d_n, d_tau = torch.zeros((L, K + 1), **i32), torch.zeros(L, **i32)
    ev, fl, fs = torch.zeros((L, N), **i32), torch.zeros((L, C), **i32), torch.zeros((L, C), **i32)
    ne, nf = torch.zeros(L, **i32), torch.zeros(L, **i32)
    r_c = np.sort(rng.random((L, K + 1)), axis=1)
    r_g = np.ascontiguousarray(np.sort(rng.random((L, K + 1)), axis=1)[:, ::-1])
    p = dict(t_cpu=40.0, t_gpu=3.0, t_io=20.0, t_draft=600.0, l_target=24, w_expert=1000, vram_left=9000)
    params = B.BalanceParams(p["t_cpu"], p["t_gpu"], p["t_io"], p["t_draft"], p["l_target"], p["w_expert"], p["vram_left"])
    d_rc, d_rg = _dev(r_c), _dev(r_g)
    z, th = np.zeros((L, N), dtype=np.int32), np.full((L, N), gamma // 2, dtype=np.int32)
    o_st = [z.copy(), z.copy(), th.copy(), th.copy()]
    o_tab = tab0.copy()
    taus, moved = set(), 0
    for t in range(steps):
        in_use = ((rng.random((L, N)) < 0.1) & (o_tab >= 0)).astype(np.int32)
        budget = rng.integers(0, 6, size=L).astype(np.int32)
        d_f = _dev(f[t])
        B.moe_utility_update(d_f, *st, d_tab, d_n, L, N, K, 1, 10)
        B.moe_balance_threshold(d_f, d_n, d_rc, d_rg, L, N, K, gamma, k, params, d_tau)
        B.moe_cache_plan(st[1], _dev(in_use), d_tab, d_tau, _dev(budget), L, N, C, K, ev, ne, fl, fs, nf)
        torch.cuda.synchronize()
        got = [x.cpu().numpy() for x in (*st, d_n, d_tau, d_tab, ev, ne, fl, fs, nf)]
        for l in range(L):
            o = oracle.utility_step(f[t, l], *(a[l] for a in o_st), K, 1, 10)
            for a, v in zip(o_st, o):
                a[l] = v
            n_tau = oracle.prefetch_counts(o_st[1][l], o_tab[l], K)
            tau = oracle.balance_threshold(f[t, l], n_tau, r_c[l], r_g[l], K, gamma, k, **p)[0]
            new, o_ev, o_fl, o_fs = oracle.cache_plan(o_st[1][l], in_use[l], o_tab[l], C, K, tau, int(budget[l]))
            o_tab[l] = new
            where = (gen, t, l)
            assert np.array_equal(got[4][l], n_tau) and got[5][l] == tau, where
            assert got[8][l] == len(o_ev) and got[11][l] == len(o_fl), where
            assert got[7][l, :len(o_ev)].tolist() == o_ev.tolist(), where
            assert got[9][l, :len(o_fl)].tolist() == o_fl.tolist() and got[10][l, :len(o_fl)].tolist() == o_fs.tolist(), where
            taus.add(tau)
            moved += len(o_fl)
        for i in range(4):
            assert np.array_equal(got[i], o_st[i]), (gen, t, i)
        assert np.array_equal(got[6], o_tab), (gen, t)
    assert moved > 0 and len(taus) > 1   # the loop moved experts and the threshold did vary


def _device_view_of_pinned(t):
    """Device address under which the GPU sees a pinned host tensor, or None when it is not mapped."""
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    dptr = ctypes.c_void_p()
    rc = hip.hipHostGetDevicePointer(ctypes.byref(dptr), ctypes.c_void_p(t.data_ptr()), 0)
    return dptr.value if rc == 0 else None


def test_pool_load_from_a_store_in_pinned_host_memory():
    """The paper's store is host memory (Sec. 3.4): experts fetched straight from pinned, device-mapped host
    memory land in their slots bit for bit; slots not named keep what they held."""
    from paper_2603_09983_amd import binding as B
    E, C, H, F = 12, 6, 128, 192
    rng = np.random.default_rng(5)
    host = [torch.from_numpy(rng.integers(-32768, 32767, size=shp, dtype=np.int16)).pin_memory()
            for shp in ((E, F, H), (E, F, H), (E, H, F))]
    for t in host:
        dv = _device_view_of_pinned(t)
        if dv is None or dv != t.data_ptr():
            pytest.skip("pinned host memory is not mapped into the device under its own address on this box")
    pools = [torch.full((C, *t.shape[1:]), 7, dtype=torch.int16, device="cuda") for t in host]
    i32 = dict(dtype=torch.int32, device="cuda")
    fetch = torch.tensor([9, 2, 11, 0, 0, 0], **i32)
    slots = torch.tensor([4, 0, 3, 0, 0, 0], **i32)
    n = torch.tensor([3], **i32)
    B.moe_pool_load(*host, *pools, fetch, slots, n, C, H, F)
    torch.cuda.synchronize()
    for t, p in zip(host, pools):
        got = p.cpu()
        for e, c in ((9, 4), (2, 0), (11, 3)):
            assert torch.equal(got[c], t[e]), (e, c)
        for c in (1, 2, 5):
            assert bool((got[c] == 7).all()), c


@pytest.mark.parametrize("H,F", [(128, 136), (8, 8), (64, 200), (256, 256), (40, 72)])
def test_pool_load_sizes_with_partial_groups(H, F):
    """Matrix sizes that are not a multiple of what a workgroup copies per round (4 x 256 words of 16 bytes),
    down to one smaller than a single wavefront's share: every word arrives, nothing else is touched."""
    from paper_2603_09983_amd import binding as B
    E, C = 7, 5
    rng = np.random.default_rng(H * 1000 + F)
    store = [_dev(rng.integers(-32768, 32767, size=shp, dtype=np.int16)) for shp in ((E, F, H), (E, F, H), (E, H, F))]
    pools = [torch.full((C + 1, *t.shape[1:]), 7, dtype=torch.int16, device="cuda") for t in store]   # one guard row
    i32 = dict(dtype=torch.int32, device="cuda")
    fetch, slots, n = torch.tensor([6, 0, 3, 0, 0], **i32), torch.tensor([2, 4, 0, 0, 0], **i32), torch.tensor([3], **i32)
    B.moe_pool_load(*store, *pools, fetch, slots, n, C, H, F)
    torch.cuda.synchronize()
    for t, p in zip(store, pools):
        for e, c in ((6, 2), (0, 4), (3, 0)):
            assert torch.equal(p[c], t[e]), (H, F, e, c)
        for c in (1, 3, 5):
            assert bool((p[c] == 7).all()), (H, F, c)
