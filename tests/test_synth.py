"""Seeded input recipes: formatting, margins and slot-table validity (host only)."""
import numpy as np
import torch

import oracle
from paper_2603_09983_amd import synth


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 0.02,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, 1e-40], np.float32)])
    ours = synth.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    back = synth.bf16_bits_to_f32(ours)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_recipes_are_deterministic_and_margined():
    for name in ("cfg1",):
        a = synth.make_layer(synth.RECIPES[name])
        b = synth.make_layer(synth.RECIPES[name])
        assert np.array_equal(a.hidden, b.hidden) and np.array_equal(a.w_down, b.w_down)
        logits = oracle.router_logits(a.hidden, a.router_w, a.router_bias)
        for t in range(a.shape.T):
            assert synth.margin_ok(logits[t], a.shape.k)
            srt = np.sort(logits[t])[::-1][: a.shape.k + 1]
            assert np.all(srt[:-1] - srt[1:] >= synth.MARGIN)


def test_slot_tables_are_injective():
    for name, r in synth.RECIPES.items():
        s = r.shape
        p = synth.zipf_popularity(r.seed, s.E, r.zipf_s) if r.zipf_s > 0 else None
        tab = synth.slot_table(r.seed, s.E, s.C, r.residency, p)
        res = tab[tab >= 0]
        assert res.size == min(s.C, s.E)
        assert np.unique(res).size == res.size and res.min() >= 0 and res.max() < s.C


def test_zipf_bias_skews_routing():
    r = synth.small_recipe("z", 9, T=64, H=64, E=16, k=2, F=32, C=4, residency="zipf", zipf_s=1.1)
    li = synth.make_layer(r)
    res = oracle.layer_from_inputs(li)
    p = synth.zipf_popularity(r.seed, 16, 1.1)
    top = np.argsort(-p)[:4]
    assert res.hist[top].sum() > res.hist.sum() * 4 / 16      # popular experts over-represented
    assert li.router_bias is not None and np.argmax(li.router_bias) == np.argmax(p)


def test_pools_are_slot_major():
    li = synth.make_layer(synth.small_recipe("p", 5, T=2, H=32, E=6, k=2, F=32, C=3))
    pg, pu, pd = li.pools()
    for e in range(6):
        c = li.slot_table[e]
        if c >= 0:
            assert np.array_equal(pg[c], li.w_gate[e]) and np.array_equal(pd[c], li.w_down[e])
