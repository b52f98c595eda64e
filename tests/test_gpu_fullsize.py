"""GPU parity at the full sizes of the named workloads, in the launch configuration the
bench times (moe_verify_layer, fp32 output).  The oracle evaluates every output of these
layers in seconds to a minute, so all outputs are compared, not a sample."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2603_09983_amd import binding as B
from paper_2603_09983_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def run_and_check(G, li, tag, form=B.LAUNCH_AUTO):
    print(f"[case] {tag} shape={li.shape}", flush=True)
    d = G.upload(li)
    buf = G.run_layer(d, form=form)
    ref = oracle.layer_from_inputs(li)
    rel = G.check_against_oracle(li, buf, ref, tag=tag)
    s = li.shape
    # properties that hold at any size
    hist = buf.hist.cpu().numpy()
    assert hist.sum() == s.T * s.k and hist.max() <= s.T
    slot_idx = buf.slot_idx.cpu().numpy().ravel()
    n = int(buf.miss_count.item())
    res = np.flatnonzero(slot_idx >= 0)
    assert np.array_equal(np.sort(np.concatenate([res, buf.miss_list.cpu().numpy()[:n]])), np.arange(s.T * s.k))
    print(f"[done] {tag} max|err|/rms = {rel:.2e} misses={n}", flush=True)
    del d, buf
    torch.cuda.empty_cache()


def test_cfg2_small_moe(G):
    run_and_check(G, synth.make_layer(synth.RECIPES["cfg2"], experts="resident"), "cfg2")


@pytest.mark.parametrize("form", ["three", "two", "one", "route+one"])
def test_cfg2_small_moe_every_launch_form(G, form):
    """Every launch form of the layer at full size (auto picks the two-launch form here; bench.py times them all)."""
    forms = {"three": B.LAUNCH_THREE, "two": B.LAUNCH_TWO, "one": B.LAUNCH_ONE, "route+one": B.LAUNCH_ROUTE_PLUS_ONE}
    run_and_check(G, synth.make_layer(synth.RECIPES["cfg2"], experts="resident"), "cfg2/" + form, form=forms[form])


def test_cfg3_fine_grained_zipf(G):
    run_and_check(G, synth.make_layer(synth.RECIPES["cfg3"], experts="resident"), "cfg3")


def test_cfg4_large_expert_both_capacities(G):
    li = synth.make_layer(synth.RECIPES["cfg4_c8"])
    run_and_check(G, li, "cfg4_c8")
    r4 = synth.RECIPES["cfg4_c4"]
    li.recipe, li.shape = r4, r4.shape
    li.slot_table = synth.slot_table(r4.seed, r4.shape.E, r4.shape.C, r4.residency)
    run_and_check(G, li, "cfg4_c4")


# the first, a middle and the last layer of the sweep's model (their residency differs) at every batch size
@pytest.mark.parametrize("layer", [0, 11, 23])
@pytest.mark.parametrize("T", [1, 5, 9, 17, 33, 64, 128])
def test_cfg5_sweep_layers(G, T, layer):
    r = synth.sweep_recipe(T, layer)
    li = synth.make_layer(r, hidden_seed=synth.sweep_hidden_seed(T), experts="resident")
    run_and_check(G, li, r.name)
