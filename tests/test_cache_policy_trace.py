"""The control loop of Sec. 3.2-3.4 run closed over long synthetic traces, oracle only (CPU):
histogram -> utility update -> cache plan -> the new slot table decides the next step's hits.

Checked at every one of the steps: what the planning step promises (never more residents than slots,
slot table one-to-one, a frozen expert keeps its slot, no unfrozen resident below tau afterwards,
no more fetches than the budget, an expert is never both evicted and fetched).  The hit rates of the
loop are compared with an LRU cache of the same capacity and per-step fetch budget and with the cache
left as it was; they are an evaluation on stand-in traces (the paper's traces need its models and
suites), printed with `pytest -s` and recorded in the design notes, and only bounded loosely here."""
import numpy as np
import pytest

import oracle
import traces


def _utility_policy(f, C, K, gamma, tau, budget, lam, frozen_rng=None, warm=50):
    steps, N = f.shape
    tab = np.full(N, -1, dtype=np.int32)
    tab[:C] = np.arange(C)
    st = (np.zeros(N, np.int32), np.zeros(N, np.int32), np.full(N, gamma // 2, np.int32), np.full(N, gamma // 2, np.int32))
    hit = tot = moved = 0
    for t in range(steps):
        if t >= warm:
            hit += int(f[t][tab >= 0].sum())
            tot += int(f[t].sum())
        st = oracle.utility_step(f[t], *st, K, *lam)
        in_use = np.zeros(N, dtype=np.int32)
        if frozen_rng is not None:
            in_use = ((frozen_rng.random(N) < 0.1) & (tab >= 0)).astype(np.int32)
        new, ev, fl, fs = oracle.cache_plan(st[1], in_use, tab, C, K, tau, budget)
        # the planning step's promises
        res = new[new >= 0]
        assert len(res) <= C and len(set(res.tolist())) == len(res) and (res < C).all(), t
        assert np.array_equal(new[in_use > 0], tab[in_use > 0]), t
        assert not ((new >= 0) & (st[1] < tau) & (in_use == 0)).any(), t
        assert len(fl) <= budget and not set(ev.tolist()) & set(fl.tolist()), t
        assert all(tab[e] >= 0 and new[e] < 0 for e in ev) and all(tab[e] < 0 and new[e] == s for e, s in zip(fl, fs)), t
        assert (st[1][fl] >= tau).all() if len(fl) else True
        tab = new
        moved += len(fl)
    return hit / max(tot, 1), moved


def _lru_policy(f, C, budget, warm=50):
    """Least-recently-used cache: after each step it loads up to `budget` of the experts that missed
    (most activated first) over the residents unused for longest."""
    steps, N = f.shape
    res = np.zeros(N, dtype=bool)
    res[:C] = True
    last = np.full(N, -1)
    hit = tot = moved = 0
    for t in range(steps):
        if t >= warm:
            hit += int(f[t][res].sum())
            tot += int(f[t].sum())
        last[f[t] > 0] = t
        missed = [e for e in np.argsort(-f[t], kind="stable") if f[t][e] > 0 and not res[e]][:budget]
        for e in missed:
            cand = np.where(res)[0]
            v = cand[np.argmin(last[cand])]
            if last[v] < t:
                res[v], res[e] = False, True
                moved += 1
    return hit / max(tot, 1), moved


TRACES = [
    # name, generator, drift, shift_every, tau
    ("smooth_drift", traces.smooth_trace, 0.1, 0, 1),
    ("smooth_with_shifts", traces.smooth_trace, 0.1, 40, 1),
    ("sampled_drift", traces.sampled_trace, 0.1, 0, 1),
    ("sampled_with_shifts", traces.sampled_trace, 0.1, 40, 2),
]


@pytest.mark.parametrize("name,gen,drift,shift,tau", TRACES, ids=[t[0] for t in TRACES])
def test_closed_loop_invariants_and_hit_rates(name, gen, drift, shift, tau):
    N, C, K, gamma, k, steps, budget = 64, 32, 4, 8, 6, 300, 4
    f = gen(np.random.default_rng(20260309), 1, N, gamma + 1, k, steps, drift, shift)[:, 0, :]
    h_util, m_util = _utility_policy(f, C, K, gamma, tau, budget, (1, 10), frozen_rng=np.random.default_rng(5))
    h_lru, m_lru = _lru_policy(f, C, budget)
    h_static = f[50:, :C].sum() / f[50:].sum()
    print(f"\n{name}: hit rate utility policy {h_util:.3f} ({m_util} loads), LRU {h_lru:.3f} ({m_lru} loads), "
          f"static {h_static:.3f}")
    assert m_util > 0 and 0.0 < h_util <= 1.0 and 0.0 < h_lru <= 1.0


def test_threshold_above_K_empties_nothing_frozen_and_fetches_nothing():
    N, C, K, gamma = 16, 8, 4, 8
    f = traces.sampled_trace(np.random.default_rng(3), 1, N, gamma + 1, 2, 40, 0.2)[:, 0, :]
    tab = np.full(N, -1, dtype=np.int32)
    tab[:C] = np.arange(C)
    st = (np.zeros(N, np.int32), np.zeros(N, np.int32), np.full(N, 4, np.int32), np.full(N, 4, np.int32))
    for t in range(40):
        st = oracle.utility_step(f[t], *st, K, 1, 10)
    frozen = np.zeros(N, dtype=np.int32)
    frozen[[1, 5]] = 1
    new, ev, fl, fs = oracle.cache_plan(st[1], frozen, tab, C, K, K + 1, N)
    assert sorted(np.where(new >= 0)[0].tolist()) == [1, 5] and len(fl) == 0 and len(ev) == C - 2
