"""Pins for the CPU oracle: what the paper and the mathematics fix.

Each `pin_*` takes an oracle.Oracle instance and raises AssertionError when
that oracle disagrees with something that does not depend on the oracle
itself: a value the paper prints (tests/golden), a closed form, an invariant,
a special case that reduces to a library routine (numpy / torch CPU), or brute
force on tiny inputs.  test_oracle_pins.py runs them on the real oracle;
test_oracle_mutants.py runs them on deliberately broken builds and requires
every planted mistake to be caught.
"""
from __future__ import annotations

import numpy as np
import scipy.special
import torch

from conftest import read_golden
from paper_2603_09983_amd import synth


# ---------------------------------------------------------------------------
# helpers that do NOT use the oracle
# ---------------------------------------------------------------------------
def bits(x):
    return synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def val(b):
    return synth.bf16_bits_to_f32(b).astype(np.float64)


def np_silu(z):
    return z * scipy.special.expit(z)


def np_expert(x, g, u, d):
    """Library evaluation of one expert on rows x: [n,H] -> [n,H] (numpy matmul, fp64)."""
    return (np_silu(x @ g.T) * (x @ u.T)) @ d.T


def rand_layer(seed, T, H, E, k, F, C, n_shared=0, Fs=0, **kw):
    r = synth.small_recipe(f"pin{seed}", seed, T=T, H=H, E=E, k=k, F=F, C=C, n_shared=n_shared,
                           F_shared=Fs, **kw)
    return synth.make_layer(r)


def dense_brute_force(li, with_shared=True):
    """Every expert on every token, multiplied by a dense [T,E] gate matrix that is
    zero outside (selected AND resident).  Selection by a full sort of each logit row."""
    s = li.shape
    x = val(li.hidden)
    logits = x @ li.router_w.astype(np.float64).T
    if li.router_bias is not None:
        logits = logits + li.router_bias.astype(np.float64)
    G = np.zeros((s.T, s.E))
    for t in range(s.T):
        order = np.lexsort((np.arange(s.E), -logits[t]))  # value desc, id asc
        sel = order[: s.k]
        p = scipy.special.softmax(logits[t])              # full softmax, then renormalise
        w = p[sel] / p[sel].sum()
        for e, we in zip(sel, w):
            if li.slot_table[e] >= 0:
                G[t, e] = we
    y = np.zeros((s.T, s.H))
    for e in range(s.E):
        y += G[:, e:e + 1] * np_expert(x, val(li.w_gate[e]), val(li.w_up[e]), val(li.w_down[e]))
    if with_shared and s.n_shared:
        for i in range(s.n_shared):
            y += np_expert(x, val(li.sh_gate[i]), val(li.sh_up[i]), val(li.sh_down[i]))
    return y


def close(a, b, tol=1e-12):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    err = np.abs(a - b)
    lim = tol * (1.0 + np.abs(b))
    assert np.all(err <= lim), f"max err {err.max():.3e}"


# ---------------------------------------------------------------------------
# step 1: router logits, top-k, gates           (Sec. 2.2)
# ---------------------------------------------------------------------------
def pin_logits_unit_vectors(O):
    """hidden = basis vector e_j  =>  logits[t,:] = W_g[:,j] (+ bias), exactly."""
    H, E = 24, 7
    rng = np.random.default_rng(1)
    W = rng.standard_normal((E, H)).astype(np.float32)
    b = rng.standard_normal(E).astype(np.float32)
    hid = np.zeros((H, H), dtype=np.float32)
    np.fill_diagonal(hid, 1.0)
    got = O.router_logits(bits(hid), W, None)
    assert np.array_equal(got, W.T.astype(np.float64))
    got = O.router_logits(bits(hid), W, b)
    assert np.array_equal(got, W.T.astype(np.float64) + b.astype(np.float64))
    # scaling one hidden entry by 2 doubles that logit contribution
    hid2 = hid.copy()
    hid2[3, 3] = 2.0
    assert np.array_equal(O.router_logits(bits(hid2), W, None)[3], 2.0 * W[:, 3].astype(np.float64))


def pin_logits_library_matmul(O):
    rng = np.random.default_rng(2)
    T, H, E = 6, 96, 11
    hid = bits(rng.standard_normal((T, H)) * 0.5)
    W = rng.standard_normal((E, H)).astype(np.float32)
    ref = val(hid) @ W.astype(np.float64).T
    close(O.router_logits(hid, W), ref, 1e-13)


def pin_topk_full_sort(O):
    """k passes of arg-max == first k of a full (value desc, id asc) sort, ties included."""
    rng = np.random.default_rng(3)
    for E, k in [(8, 2), (64, 6), (60, 4), (5, 5), (9, 1), (130, 7)]:
        logits = np.round(rng.standard_normal((40, E)) * 2.0) / 2.0  # heavy ties
        idx, _ = O.topk_gate(logits, k)
        for t in range(logits.shape[0]):
            order = np.lexsort((np.arange(E), -logits[t]))
            assert np.array_equal(idx[t], order[:k]), (E, k, t)


def pin_topk_special_cases(O):
    rng = np.random.default_rng(4)
    logits = rng.standard_normal((10, 12))
    idx, g = O.topk_gate(logits, 1)
    assert np.array_equal(idx[:, 0], logits.argmax(axis=1))
    assert np.all(g == 1.0)                                     # k=1 => weight exactly 1
    idx, g = O.topk_gate(logits, 12)
    assert np.array_equal(np.sort(idx, axis=1), np.tile(np.arange(12), (10, 1)))  # permutation
    flat = np.zeros((3, 9))
    idx, g = O.topk_gate(flat, 4)
    assert np.array_equal(idx, np.tile(np.arange(4), (3, 1)))   # ties -> lower id
    assert np.all(g == 0.25)                                    # equal logits -> 1/k


def pin_gate_closed_forms(O):
    gold = read_golden("logistic_constants.txt")["gate_top2_of_ln4_ln1_ln2_ln3"]
    logits = np.log(np.array([[4.0, 1.0, 2.0, 3.0]]))
    idx, g = O.topk_gate(logits, 2)
    assert idx[0].tolist() == [int(gold[0]), int(gold[1])]
    close(g[0], [float(gold[2]), float(gold[3])], 1e-15)
    # sum to one, shift invariance, equality with softmax-over-all then renormalise
    rng = np.random.default_rng(5)
    logits = rng.standard_normal((50, 64)) * 3.0
    idx, g = O.topk_gate(logits, 6)
    close(g.sum(axis=1), np.ones(50), 1e-15)
    idx2, g2 = O.topk_gate(logits + 123.25, 6)
    assert np.array_equal(idx, idx2)
    close(g2, g, 1e-12)
    p = scipy.special.softmax(logits, axis=1)
    sel = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    close(g, sel / sel.sum(axis=1, keepdims=True), 1e-13)
    assert np.all(np.diff(g, axis=1) <= 0)  # listed by descending logit


# ---------------------------------------------------------------------------
# step 2: activation frequency               (Sec. 2.3)
# ---------------------------------------------------------------------------
def _worked_example():
    g = read_golden("worked_example_appC1.txt")
    E, k = int(g["num_experts"][0]), int(g["top_k"][0])
    toks = " ".join(g["token_experts"]).split(";")
    idx = np.array([[int(v) for v in t.split()] for t in toks], dtype=np.int32)
    table = np.full(E, -1, dtype=np.int32)
    for c, e in enumerate(g["resident"]):
        table[int(e)] = c
    return g, E, k, idx, table


def pin_hist_worked_example(O):
    g, E, k, idx, table = _worked_example()
    hist = O.expert_histogram(idx, E)
    assert hist.tolist() == [int(v) for v in g["hist"]]
    assert int((hist > 0).sum()) == int(g["distinct_active"][0])
    assert int(((hist > 0) & (table >= 0)).sum()) == int(g["distinct_active_resident"][0])
    assert abs(((hist > 0) & (table >= 0)).sum() / (hist > 0).sum() - float(g["r_g"][0])) < 1e-15


def pin_hist_invariants(O):
    rng = np.random.default_rng(6)
    for T, E, k in [(1, 64, 6), (9, 64, 6), (5, 8, 2), (128, 64, 6), (3, 4, 4)]:
        logits = rng.standard_normal((T, E))
        idx, _ = O.topk_gate(logits, k)
        hist = O.expert_histogram(idx, E)
        assert hist.sum() == T * k
        assert hist.min() >= 0 and hist.max() <= T       # range of f: [0, gamma+1]
        assert (hist > 0).sum() <= min(E, T * k)          # b <= gamma*k
        if T == 1:
            assert sorted(hist.tolist()) == [0] * (E - k) + [1] * k   # binary signal at T=1
        assert np.array_equal(hist, np.bincount(idx.ravel(), minlength=E))
    # a hand-made case with a repeated expert inside the batch but a quiet expert too
    idx = np.array([[5, 1], [5, 2], [1, 5]], dtype=np.int32)
    assert O.expert_histogram(idx, 7).tolist() == [0, 2, 1, 0, 0, 3, 0]


# ---------------------------------------------------------------------------
# step 3: slot resolve and miss list            (App. D)
# ---------------------------------------------------------------------------
def pin_slot_worked_example(O):
    g, E, k, idx, table = _worked_example()
    slot_idx, miss, n = O.slot_resolve(idx, table)
    assert n == int(g["missed_assignments"][0])
    assert (slot_idx >= 0).sum() == int(g["resident_assignments"][0])
    assert sorted(set(idx.ravel()[miss].tolist())) == [int(v) for v in g["missed_experts"]]
    assert abs(n / idx.size - float(g["r_c"][0])) < 1e-15
    assert miss.tolist() == [0, 2]                        # flat ids t*k+j, ascending
    assert slot_idx.tolist() == [[-1, 0], [-1, 0]]


def pin_slot_partition(O):
    rng = np.random.default_rng(7)
    T, E, k, C = 17, 64, 6, 20
    idx, _ = O.topk_gate(rng.standard_normal((T, E)), k)
    table = np.full(E, -1, dtype=np.int32)
    chosen = rng.choice(E, C, replace=False)
    table[chosen] = rng.permutation(C)
    slot_idx, miss, n = O.slot_resolve(idx, table)
    flat = slot_idx.ravel()
    res = np.flatnonzero(flat >= 0)
    assert n + res.size == T * k
    assert np.array_equal(np.sort(np.concatenate([res, miss])), np.arange(T * k))
    assert np.all(np.diff(miss) > 0)
    assert np.array_equal(flat, table[idx.ravel()])
    # identity table: nothing missed; empty table: everything missed
    s2, m2, n2 = O.slot_resolve(idx, np.arange(E, dtype=np.int32))
    assert n2 == 0 and np.array_equal(s2, idx)
    s3, m3, n3 = O.slot_resolve(idx, np.full(E, -1, dtype=np.int32))
    assert n3 == T * k and np.all(s3 == -1) and np.array_equal(m3, np.arange(T * k))
    # relabelling the slots changes slot ids only
    perm = rng.permutation(C).astype(np.int32)
    t2 = table.copy()
    t2[table >= 0] = perm[table[table >= 0]]
    s4, m4, n4 = O.slot_resolve(idx, t2)
    assert np.array_equal(m4, miss) and np.array_equal(s4 >= 0, slot_idx >= 0)
    assert np.array_equal(s4[slot_idx >= 0], perm[slot_idx[slot_idx >= 0]])


# ---------------------------------------------------------------------------
# step 4: expert FFN and weighted combine      (Sec. 2.2 last line; App. D)
# ---------------------------------------------------------------------------
def pin_ffn_closed_form(O):
    """x = e_0, W_gate[:,0] = a, W_up[:,0] = b, W_down a known 2x3 matrix  =>
    y = W_down (silu(a) * b) with silu from the golden logistic constants."""
    c = read_golden("logistic_constants.txt")
    silu = {1.0: float(c["silu(1)"][0]), -1.0: float(c["silu(-1)"][0]), 2.0: float(c["silu(2)"][0])}
    H, F = 2, 3
    a = [1.0, -1.0, 2.0]
    b = [0.5, 4.0, -3.0]
    wg = np.zeros((1, F, H), dtype=np.float32); wg[0, :, 0] = a; wg[0, :, 1] = 7.0   # column 1 unused by x
    wu = np.zeros((1, F, H), dtype=np.float32); wu[0, :, 0] = b; wu[0, :, 1] = -5.0
    wd = np.array([[[1.0, 2.0, 0.0], [0.0, 0.0, 1.0]]], dtype=np.float32)            # [1,H,F]
    x = np.array([[1.0, 0.0]], dtype=np.float32)
    idx = np.zeros((1, 1), dtype=np.int32)
    gate = np.ones((1, 1))
    y = O.routed_ffn(bits(x), idx, gate, np.zeros(1, np.int32), bits(wg), bits(wu), bits(wd))
    m = [silu[a[i]] * b[i] for i in range(3)]
    close(y[0], [m[0] + 2.0 * m[1], m[2]], 1e-15)
    # gate weight scales the result; a non-resident expert contributes nothing
    y2 = O.routed_ffn(bits(x), idx, gate * 0.25, np.zeros(1, np.int32), bits(wg), bits(wu), bits(wd))
    close(y2, 0.25 * y, 1e-15)
    y3 = O.routed_ffn(bits(x), idx, gate, np.full(1, -1, np.int32), bits(wg), bits(wu), bits(wd))
    assert np.all(y3 == 0.0)


def pin_ffn_textbook_swiglu(O):
    """E = k = 1: the layer is a plain SwiGLU MLP; compare with torch's own linear + silu."""
    rng = np.random.default_rng(8)
    T, H, F = 4, 48, 80
    x = bits(rng.standard_normal((T, H)) * 0.7)
    wg = bits(rng.standard_normal((1, F, H)) * 0.3)
    wu = bits(rng.standard_normal((1, F, H)) * 0.3)
    wd = bits(rng.standard_normal((1, H, F)) * 0.3)
    res = O.verify_layer(x, rng.standard_normal((1, H)).astype(np.float32), None, np.zeros(1, np.int32),
                         wg, wu, wd, 1)
    tx = torch.from_numpy(val(x))
    ref = torch.nn.functional.linear(
        torch.nn.functional.silu(torch.nn.functional.linear(tx, torch.from_numpy(val(wg[0]))))
        * torch.nn.functional.linear(tx, torch.from_numpy(val(wu[0]))),
        torch.from_numpy(val(wd[0]))).numpy()
    assert np.all(res.gate == 1.0) and np.all(res.topk_idx == 0)
    close(res.y, ref, 1e-12)


def pin_ffn_dense_brute_force(O):
    for seed, kw in [(21, dict(T=5, H=32, E=8, k=2, F=48, C=8, residency="all")),
                     (22, dict(T=7, H=64, E=12, k=3, F=32, C=5)),
                     (23, dict(T=4, H=32, E=10, k=4, F=64, C=4, n_shared=2, Fs=32)),
                     (24, dict(T=6, H=32, E=9, k=3, F=32, C=4, n_shared=1, Fs=96, zipf_s=1.1,
                               residency="zipf"))]:
        li = rand_layer(seed, **kw)
        res = O.layer_from_inputs(li)
        close(res.y, dense_brute_force(li), 1e-12)


def pin_ffn_identical_experts(O):
    """All experts share one weight set: all resident => y_t = FFN(x_t) whatever the
    router picks (gates sum to 1); partial cache => y_t = (sum of resident gates) FFN(x_t)."""
    li = rand_layer(31, T=6, H=32, E=8, k=3, F=48, C=8, residency="all")
    for e in range(1, 8):
        li.w_gate[e], li.w_up[e], li.w_down[e] = li.w_gate[0], li.w_up[0], li.w_down[0]
    ffn = np_expert(val(li.hidden), val(li.w_gate[0]), val(li.w_up[0]), val(li.w_down[0]))
    res = O.layer_from_inputs(li)
    close(res.y, ffn, 1e-12)
    li.slot_table[:] = -1
    li.slot_table[[1, 4, 6]] = [2, 0, 1]
    res = O.layer_from_inputs(li)
    wsum = (res.gate * (res.slot_idx >= 0)).sum(axis=1, keepdims=True)
    close(res.y, wsum * ffn, 1e-12)


def pin_ffn_linearity_and_symmetry(O):
    li = rand_layer(41, T=6, H=32, E=10, k=3, F=32, C=4)
    full = li.slot_table.copy()
    res_a = O.layer_from_inputs(li)
    comp = np.full_like(full, -1)
    comp[full < 0] = np.arange((full < 0).sum())
    li.slot_table = comp
    res_b = O.layer_from_inputs(li)
    li.slot_table = np.arange(li.shape.E, dtype=np.int32)
    res_all = O.layer_from_inputs(li)
    close(res_a.y + res_b.y, res_all.y, 1e-12)          # device part + host part = whole
    assert res_a.miss_count + res_b.miss_count == li.shape.T * li.shape.k
    li.slot_table = full
    # token permutation equivariance
    perm = np.random.default_rng(0).permutation(li.shape.T)
    hid0 = li.hidden.copy()
    li.hidden = hid0[perm]
    res_p = O.layer_from_inputs(li)
    li.hidden = hid0
    close(res_p.y, res_a.y[perm], 1e-13)
    assert np.array_equal(res_p.topk_idx, res_a.topk_idx[perm])
    # expert relabelling invariance (permute router rows, weights and table together)
    q = np.random.default_rng(1).permutation(li.shape.E)
    li2 = rand_layer(41, T=6, H=32, E=10, k=3, F=32, C=4)
    li2.router_w, li2.slot_table = li.router_w[q], li.slot_table[q]
    li2.w_gate, li2.w_up, li2.w_down = li.w_gate[q], li.w_up[q], li.w_down[q]
    res_q = O.layer_from_inputs(li2)
    close(res_q.y, res_a.y, 1e-12)
    assert np.array_equal(q[res_q.topk_idx], res_a.topk_idx)
    assert np.array_equal(res_q.hist, res_a.hist[q])


def pin_ffn_zero_cases(O):
    li = rand_layer(51, T=3, H=32, E=6, k=2, F=32, C=6, residency="all")
    wd = li.w_down.copy()
    li.w_down = np.zeros_like(wd)
    assert np.all(O.layer_from_inputs(li).y == 0.0)
    li.w_down = wd
    li.hidden = np.zeros_like(li.hidden)
    assert np.all(O.layer_from_inputs(li).y == 0.0)


def pin_shared_experts(O):
    """Shared experts add E_s(x_t) with weight 1 for every token, and two shared experts
    of width F equal one of width 2F (concatenate gate/up rows, down columns)."""
    li = rand_layer(61, T=5, H=32, E=6, k=2, F=32, C=3, n_shared=2, Fs=48)
    x = val(li.hidden)
    y0 = np.zeros((5, 32))
    O.shared_ffn_add(li.hidden, li.sh_gate, li.sh_up, li.sh_down, y0)
    ref = sum(np_expert(x, val(li.sh_gate[i]), val(li.sh_up[i]), val(li.sh_down[i])) for i in range(2))
    close(y0, ref, 1e-12)
    cat_g = np.concatenate([li.sh_gate[0], li.sh_gate[1]], axis=0)[None]
    cat_u = np.concatenate([li.sh_up[0], li.sh_up[1]], axis=0)[None]
    cat_d = np.concatenate([li.sh_down[0], li.sh_down[1]], axis=1)[None]
    y1 = np.zeros((5, 32))
    O.shared_ffn_add(li.hidden, cat_g, cat_u, cat_d, y1)
    close(y1, y0, 1e-12)
    # whole layer = routed part + shared part; shared experts are outside hist and miss list
    res = O.layer_from_inputs(li)
    routed = O.routed_ffn(li.hidden, res.topk_idx, res.gate, li.slot_table, li.w_gate, li.w_up, li.w_down)
    close(res.y, routed + y0, 1e-13)
    assert res.hist.sum() == li.shape.T * li.shape.k


def pin_layer_composition(O):
    li = rand_layer(71, T=9, H=64, E=16, k=4, F=32, C=8)
    res = O.layer_from_inputs(li)
    logits = O.router_logits(li.hidden, li.router_w, li.router_bias)
    idx, gate = O.topk_gate(logits, li.shape.k)
    assert np.array_equal(res.logits, logits) and np.array_equal(res.topk_idx, idx)
    assert np.array_equal(res.gate, gate)
    assert np.array_equal(res.hist, O.expert_histogram(idx, li.shape.E))
    s, m, n = O.slot_resolve(idx, li.slot_table)
    assert np.array_equal(res.slot_idx, s) and np.array_equal(res.miss_list, m) and res.miss_count == n
    assert np.array_equal(res.y, O.routed_ffn(li.hidden, idx, gate, li.slot_table, li.w_gate, li.w_up,
                                              li.w_down))


ALL_PINS = [v for k, v in sorted(globals().items()) if k.startswith("pin_")]


# ---------------------------------------------------------------------------
# Speculative Utility Estimator (Sec. 3.2, Alg. 1) and n(tau) (Sec. 3.3)
# ---------------------------------------------------------------------------
def _est_init(N, gamma):
    z = np.zeros(N, dtype=np.int32)
    th = np.full(N, gamma // 2, dtype=np.int32)
    return z.copy(), z.copy(), th.copy(), th.copy()   # f_prev, s, th_up, th_dn


def pin_est_hand_trace(O):
    """The pencil trace in tests/golden/utility_trace_alg1.txt (gamma = 4, lambda = 1/2)."""
    import os
    from conftest import GOLDEN
    with open(os.path.join(GOLDEN, "utility_trace_alg1.txt")) as fh:
        rows = [l.split("#")[0].split() for l in fh]
    rows = [r for r in rows if r]
    assert len(rows) == 14
    state = {}
    for name, K, f, s1, up1, dn1 in rows:
        if name not in state:
            state[name] = _est_init(1, 4)
        fp, s, up, dn = state[name]
        fp, s, up, dn = O.utility_step(np.array([int(f)], dtype=np.int32), fp, s, up, dn, int(K), 1, 2)
        state[name] = (fp, s, up, dn)
        assert (int(s[0]), int(up[0]), int(dn[0])) == (int(s1), int(up1), int(dn1)), (name, f, s, up, dn)
        assert int(fp[0]) == int(f)


def pin_est_closed_forms(O):
    """lambda = 0 freezes the boundaries, which gives closed forms: a constant frequency never moves
    the utility; a ramp of slope >= boundary reaches min(K, t); a square wave of height >= boundary
    alternates 1, 0; and a slope one below the boundary never moves it."""
    N, gamma, K = 4, 6, 5
    th = gamma // 2
    fp, s, up, dn = _est_init(N, gamma)
    for t in range(1, 12):
        f = np.array([7, th * t, (t % 2) * th, (th - 1) * t], dtype=np.int32)
        fp, s, up, dn = O.utility_step(f, fp, s, up, dn, K, 0, 10)
        want0 = 1 if 7 >= th else 0              # the jump 0 -> 7 at t = 1 counts once, then d = 0
        assert s[0] == want0 and s[1] == min(K, t) and s[2] == t % 2 and s[3] == 0, (t, s)
        assert np.all(up == th) and np.all(dn == th)
    # lambda = 1: the boundary becomes the last fluctuation of its sign
    fp, s, up, dn = _est_init(1, 6)
    for f, eu, ed in ((5, 5, 3), (7, 2, 3), (1, 2, 6), (1, 2, 6), (0, 2, 1)):
        fp, s, up, dn = O.utility_step(np.array([f], dtype=np.int32), fp, s, up, dn, 4, 1, 1)
        assert (up[0], dn[0]) == (eu, ed), (f, up, dn)


def pin_est_zero_boundary_and_floor(O):
    """gamma = 1 starts the boundaries at 0: the upward test d >= 0 then holds for d = 0 too, so a
    constant frequency climbs to K (the listing's '>=', upward test first).  And the floor is exact:
    boundary 10 with fluctuation +10 at lambda = 1/10 stays 10; 3 with +7 gives floor(3.4) = 3; 1
    with -1 stays floor(0.9 + 0.1) = 1 (never reaches 0 through calibration)."""
    fp, s, up, dn = _est_init(1, 1)
    for t in range(1, 6):
        fp, s, up, dn = O.utility_step(np.array([0], dtype=np.int32), fp, s, up, dn, 3, 1, 10)
        assert s[0] == min(3, t) and up[0] == 0 and dn[0] == 0
    for th0, d, want in ((10, 10, 10), (3, 7, 3), (9, 19, 10), (1, 1, 1), (29, 1, 26)):
        fp = np.array([100], dtype=np.int32)
        s = np.array([2], dtype=np.int32)
        up = np.array([th0], dtype=np.int32)
        dn = np.array([th0], dtype=np.int32)
        _, _, up2, dn2 = O.utility_step(np.array([100 + d], dtype=np.int32), fp, s, up, dn, 4, 1, 10)
        assert up2[0] == want and dn2[0] == th0, (th0, d, up2, dn2)
        _, _, up3, dn3 = O.utility_step(np.array([100 - d], dtype=np.int32), fp, s, up, dn, 4, 1, 10)
        assert dn3[0] == want and up3[0] == th0, (th0, d, up3, dn3)


def pin_est_invariants(O):
    """On random frequency sequences: 0 <= s <= K and |s_{t+1} - s_t| <= 1; the boundary on the side
    of the fluctuation lands between its old value and |d| (a convex combination, floored), the
    other one is untouched; d = 0 with positive boundaries changes nothing; experts do not
    interact (running them one at a time gives the same states); f_prev follows f."""
    rng = np.random.default_rng(7)
    N, gamma, K = 16, 8, 4
    fp, s, up, dn = _est_init(N, gamma)
    solo = [_est_init(1, gamma) for _ in range(N)]
    for t in range(60):
        f = rng.integers(0, gamma + 2, size=N).astype(np.int32)
        if t % 7 == 3:
            f = fp.copy()
        d = f.astype(np.int64) - fp
        fp2, s2, up2, dn2 = O.utility_step(f, fp, s, up, dn, K, 1, 10)
        assert np.all(s2 >= 0) and np.all(s2 <= K) and np.all(np.abs(s2 - s) <= 1)
        pos, neg, zero = d > 0, d < 0, d == 0
        assert np.all(up2[~pos] == up[~pos]) and np.all(dn2[~neg] == dn[~neg])
        assert np.all(up2[pos] >= np.minimum(up[pos], d[pos])) and np.all(up2[pos] <= np.maximum(up[pos], d[pos]))
        assert np.all(dn2[neg] >= np.minimum(dn[neg], -d[neg])) and np.all(dn2[neg] <= np.maximum(dn[neg], -d[neg]))
        still = zero & (up > 0)
        assert np.all(s2[still] == s[still])
        assert np.all(s2[d >= up] == np.minimum(K, s[d >= up] + 1))
        assert np.array_equal(fp2, f)
        for i in range(N):
            solo[i] = O.utility_step(f[i:i + 1], *solo[i], K, 1, 10)
            assert (solo[i][1][0], solo[i][2][0], solo[i][3][0]) == (s2[i], up2[i], dn2[i])
        fp, s, up, dn = fp2, s2, up2, dn2


def pin_prefetch_counts(O):
    """n(tau) by brute force with numpy, its monotonicity in tau, and the worked example of
    App. C.1 read as utilities: resident set {3}, so every other hot expert must be fetched."""
    rng = np.random.default_rng(3)
    for N, K in ((8, 4), (64, 4), (130, 7)):
        s = rng.integers(0, K + 1, size=N).astype(np.int32)
        tab = np.where(rng.random(N) < 0.4, np.arange(N), -1).astype(np.int32)
        n = O.prefetch_counts(s, tab, K)
        want = np.array([int(np.sum((s >= tau) & (tab < 0))) for tau in range(K + 1)])
        assert np.array_equal(n, want)
        assert n[0] == int(np.sum(tab < 0)) and np.all(np.diff(n) <= 0)
    s = np.array([1, 0, 1, 2], dtype=np.int32)
    tab = np.array([-1, -1, -1, 0], dtype=np.int32)
    assert np.array_equal(O.prefetch_counts(s, tab, 2), [3, 2, 0])


ALL_PINS = [v for k, v in sorted(globals().items()) if k.startswith("pin_")]


# ---------------------------------------------------------------------------
# Heterogeneous Workload Balancer (Sec. 3.3; appendix on its formulation)
# ---------------------------------------------------------------------------
_BAL = dict(t_cpu=40.0, t_gpu=3.0, t_io=25.0, t_draft=600.0, l_target=24, w_expert=17_301_504, vram_left=10**12)


def _bal(O, f, n_tau, r_c, r_g, K, gamma, k, **kw):
    p = dict(_BAL)
    p.update(kw)
    return O.balance_threshold(f, n_tau, r_c, r_g, K, gamma, k, **p)


def pin_balancer_worked_example(O):
    """App. C.1: gamma = 2, k = 2, resident {3}, tokens {0,3},{2,3}: r_c = 1/2, b = 3, r_g = 1/3, so
    the host takes r_c * 4 = 2 unit times and the device r_g * 3 = 1 unit time."""
    g = _worked_example()[0]
    hist = np.array([int(v) for v in g["hist"]], dtype=np.int32)
    r_c = np.array([0.0, float(g["r_c"][0])])
    r_g = np.array([0.0, float(g["r_g"][0])])
    tau, b, tc, tg = _bal(O, hist, np.zeros(2, dtype=np.int32), r_c, r_g, 1, 2, 2, t_cpu=7.0, t_gpu=5.0)
    assert b == 3 == int(g["distinct_active"][0]) and tau == 1
    close(tc[1], 2 * 7.0)
    close(tg[1], 1 * 5.0)


def _four_candidates(tc, tg, feas, K):
    """The appendix's shortcut, written independently: feasible bounds, and floor / ceil of the point
    where the two (linearly interpolated) time curves cross; smaller tau on ties; K if infeasible."""
    S = [t for t in range(1, K + 1) if feas[t]]
    if not S:
        return K
    cand = {S[0], S[-1]}
    d = tc - tg
    for t in range(1, K):
        if d[t] == 0:
            cand.add(t)
        if d[t] * d[t + 1] < 0:
            cross = t + d[t] / (d[t] - d[t + 1])
            cand.update({int(np.floor(cross)), int(np.ceil(cross))})
    if d[K] == 0:
        cand.add(K)
    cand = sorted(c for c in cand if c in S)
    return min(cand, key=lambda t: (abs(d[t]), t))


def pin_balancer_convex_shortcut(O):
    """With r_c increasing and r_g decreasing in tau (the paper's premise) and a contiguous feasible
    range, evaluating every tau and the four-candidate shortcut agree."""
    rng = np.random.default_rng(11)
    for trial in range(200):
        K = int(rng.integers(1, 9))
        gamma, k = int(rng.integers(K, 16)), int(rng.integers(1, 9))
        r_c = np.concatenate([[0.0], np.sort(rng.random(K))])
        r_g = np.concatenate([[1.0], np.sort(rng.random(K))[::-1]])
        N = 64
        f = (rng.random(N) < 0.3).astype(np.int32) * rng.integers(1, gamma + 2, size=N).astype(np.int32)
        n_tau = np.concatenate([[40], np.sort(rng.integers(0, 40, size=K))[::-1]]).astype(np.int32)
        kw = dict(t_cpu=float(rng.uniform(5, 80)), t_gpu=float(rng.uniform(0.5, 10)),
                  t_io=float(rng.uniform(1, 60)), t_draft=float(rng.uniform(100, 900)))
        tau, b, tc, tg = _bal(O, f, n_tau, r_c, r_g, K, gamma, k, **kw)
        assert b == int((f > 0).sum())
        win = np.maximum(tc, tg) + gamma * kw["t_draft"] / _BAL["l_target"]
        feas = np.zeros(K + 1, dtype=bool)
        feas[1:] = kw["t_io"] * n_tau[1:] <= win[1:]
        S = np.flatnonzero(feas)
        if len(S) and S[-1] - S[0] + 1 != len(S):
            continue   # (n(tau) decreasing makes the feasible set an upper range; skip oddities of random draws)
        assert tau == _four_candidates(tc, tg, feas, K), (trial, tau, tc, tg, feas)


def pin_balancer_constraints_and_limits(O):
    """Closed cases: an idle host (t_cpu = 0) sends everything above the largest feasible threshold
    to it; an idle device the smallest; the I/O and the memory limits each cut the range from below
    ('<=' holds with equality); nothing feasible gives K; scaling every time by 8 changes nothing."""
    K, gamma, k = 4, 8, 6
    f = np.array([3, 0, 1, 2, 0, 9], dtype=np.int32)             # b = 4
    r_c = np.array([0.0, 0.1, 0.3, 0.6, 0.9])
    r_g = np.array([1.0, 0.9, 0.7, 0.4, 0.2])
    n_tau = np.array([6, 5, 3, 2, 0], dtype=np.int32)
    assert _bal(O, f, n_tau, r_c, r_g, K, gamma, k, t_cpu=0.0)[0] == 4
    assert _bal(O, f, n_tau, r_c, r_g, K, gamma, k, t_gpu=0.0)[0] == 1
    tau0, b, tc, tg = _bal(O, f, n_tau, r_c, r_g, K, gamma, k)
    assert b == 4
    want = min(range(1, K + 1), key=lambda t: (abs(r_c[t] * gamma * k * 40.0 - r_g[t] * 4 * 3.0), t))
    assert tau0 == want
    # memory: room for exactly n(2) = 3 experts -> tau = 1 (5 experts) is out, tau = 2 is in
    w = _BAL["w_expert"]
    assert _bal(O, f, n_tau, r_c, r_g, K, gamma, k, t_gpu=0.0, vram_left=3 * w)[0] == 2
    assert _bal(O, f, n_tau, r_c, r_g, K, gamma, k, t_gpu=0.0, vram_left=3 * w - 1)[0] == 3
    # I/O: window(tau) = max(Tc,Tg) + gamma*t_draft/L; choose t_io so that tau = 1 sits exactly on the limit
    win1 = max(tc[1], tg[1]) + gamma * 600.0 / 24
    assert _bal(O, f, n_tau, r_c, r_g, K, gamma, k, t_gpu=0.0, t_io=win1 / 5 * (1 + 1e-9))[0] >= 2
    tc0 = r_c[1] * gamma * k * 40.0
    assert _bal(O, f, n_tau, r_c, r_g, K, gamma, k, t_gpu=0.0, t_io=(tc0 + gamma * 600.0 / 24) / 5)[0] == 1
    # nothing feasible -> K
    assert _bal(O, f, np.array([6, 5, 5, 5, 5], dtype=np.int32), r_c, r_g, K, gamma, k, vram_left=w)[0] == K
    # tie -> smaller tau
    r_sym = np.array([0.0, 0.2, 0.2, 0.2, 0.2])
    assert _bal(O, f, np.zeros(5, dtype=np.int32), r_sym, r_sym, K, gamma, k)[0] == 1
    s8 = _bal(O, f, n_tau, r_c, r_g, K, gamma, k, t_cpu=320.0, t_gpu=24.0, t_io=200.0, t_draft=4800.0)
    assert s8[0] == tau0
    close(s8[2][1:], 8 * tc[1:])
    close(s8[3][1:], 8 * tg[1:])


ALL_PINS = [v for k, v in sorted(globals().items()) if k.startswith("pin_")]


# ---------------------------------------------------------------------------
# Utility-guided cache manager, one planning step (Sec. 3.4; appendix on the engine)
# ---------------------------------------------------------------------------
def pin_cache_plan_hand_example(O):
    g = read_golden("cache_plan_example.txt")
    ints = lambda k: np.array([int(v) for v in g[k]], dtype=np.int32)
    tab, ev, fl, fs = O.cache_plan(ints("utility"), ints("in_use"), ints("slot_before"), 4, 4, 2, 3)
    assert ev.tolist() == ints("evict").tolist() and fl.tolist() == ints("fetch").tolist()
    assert fs.tolist() == ints("fetch_slot").tolist() and tab.tolist() == ints("slot_after").tolist()
    # a budget of one fetch takes only the first request of the highest level
    tab, ev, fl, fs = O.cache_plan(ints("utility"), ints("in_use"), ints("slot_before"), 4, 4, 2, 1)
    assert fl.tolist() == [0] and fs.tolist() == [0] and tab.tolist() == [0, -1, 1, -1, 3, -1, -1, -1]


def pin_cache_plan_invariants_and_sorted_reference(O):
    """Random states: frozen experts are never evicted; exactly the unfrozen residents below tau are;
    the table stays one-to-one and within C; what is fetched is the head of the candidates sorted by
    (utility descending, id ascending) by a library sort, cut at the free slots and the budget; slots
    are handed out ascending; nothing is both evicted and fetched; every unfrozen resident after the
    step has utility >= tau."""
    rng = np.random.default_rng(17)
    for trial in range(300):
        N, K = int(rng.integers(1, 40)), int(rng.integers(1, 7))
        C = int(rng.integers(0, N + 3))
        s = rng.integers(0, K + 1, size=N).astype(np.int32)
        tab = np.full(N, -1, dtype=np.int32)
        res = rng.permutation(N)[:int(rng.integers(0, min(N, C) + 1))]
        tab[res] = rng.permutation(C)[:len(res)]
        in_use = ((rng.random(N) < 0.2) & (tab >= 0)).astype(np.int32)
        tau, budget = int(rng.integers(0, K + 2)), int(rng.integers(0, N + 1))
        new, ev, fl, fs = O.cache_plan(s, in_use, tab, C, K, tau, budget)
        want_ev = sorted([i for i in range(N) if tab[i] >= 0 and not in_use[i] and s[i] < tau], key=lambda i: (s[i], i))
        assert ev.tolist() == want_ev
        kept = [i for i in range(N) if tab[i] >= 0 and i not in want_ev]
        free = sorted(set(range(C)) - {int(tab[i]) for i in kept})
        cand = sorted([i for i in range(N) if (tab[i] < 0 or i in want_ev) and tau <= s[i] <= K], key=lambda i: (-s[i], i))
        # (an expert evicted in this step has utility < tau, so it is never a candidate)
        n = min(len(cand), len(free), budget)
        assert fl.tolist() == cand[:n] and fs.tolist() == free[:n]
        want = tab.copy()
        want[want_ev] = -1
        want[cand[:n]] = free[:n]
        assert np.array_equal(new, want)
        held = new[new >= 0]
        assert len(set(held.tolist())) == len(held) and (len(held) == 0 or held.max() < C)
        assert all(s[i] >= tau or in_use[i] for i in range(N) if new[i] >= 0)
        assert not set(ev.tolist()) & set(fl.tolist())


ALL_PINS = [v for k, v in sorted(globals().items()) if k.startswith("pin_")]
