"""The failure path of the bounded waits, forced from the host: with a poll limit of a few polls and a skew of
one between the call number that producers stamp and the one that consumers look for, no wait inside a launch
ever finds its entry.  Every kernel must still end by itself, the call must mark its results (NaN in `out`,
-1 in miss_count), moe_workspace_status must report it, and the next call on the same workspace, without a new
moe_workspace_init, must be right again (the status call steps the call counter past the failed call's numbers)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_09983_amd import binding as B
from paper_2603_09983_amd import synth

pytestmark = pytest.mark.gpu

FORMS = {"three": B.LAUNCH_THREE, "two": B.LAUNCH_TWO, "one": B.LAUNCH_ONE, "route+one": B.LAUNCH_ROUTE_PLUS_ONE}


def _call(d, buf, form, check=True):
    return B.moe_verify_layer(B.with_form(d.shape, form), d.hidden, d.router_w, d.router_bias, d.slot_table, d.w_gate,
                              d.w_up, d.w_down, d.sh_gate, d.sh_up, d.sh_down, buf.topk_idx, buf.topk_w, buf.hist,
                              buf.slot_idx, buf.miss_list, buf.miss_count, buf.out, False, False, buf.workspace,
                              check=check)


@pytest.mark.parametrize("case,forms", [
    ("small", ("three", "two", "one", "route+one")),   # T <= 32: the final sum waits inside the down kernel
    ("cfg2", ("three", "two", "one", "route+one")),
    ("two_groups", ("three", "two")),                  # 17-32 tokens: two tokens per wavefront in the routing steps
    ("separate_sum", ("three", "two")),                # 24 tokens whose strip of the final sum does not fit the down
                                                       # kernel's tile buffer: a kernel of its own sums, and marks
    ("wide", ("three",)),                              # T > 32: a kernel of its own does the final sum
])
def test_a_wait_that_runs_out_is_reported_and_recovered_from(case, forms):
    import gpu_util as G
    if case == "cfg2":
        li = synth.make_layer(synth.RECIPES["cfg2"], experts="resident")
    elif case == "small":
        li = synth.make_layer(synth.small_recipe("wait_small", 4711, T=6, H=256, E=16, k=4, F=128, C=12,
                                                 n_shared=1, F_shared=128))
    elif case == "two_groups":
        li = synth.make_layer(synth.small_recipe("wait_two_groups", 4713, T=24, H=256, E=16, k=4, F=128, C=12,
                                                 n_shared=1, F_shared=128))
    elif case == "separate_sum":
        li = synth.make_layer(synth.small_recipe("wait_separate_sum", 4714, T=24, H=256, E=64, k=8, F=64, C=45,
                                                 n_shared=3, F_shared=192, hidden="unit"))
    else:
        li = synth.make_layer(synth.small_recipe("wait_wide", 4712, T=40, H=256, E=16, k=4, F=128, C=12,
                                                 n_shared=1, F_shared=128))
    d = G.upload(li)
    ref = oracle.layer_from_inputs(li)
    for fname in forms:
        form = FORMS[fname]
        buf = B.LayerBuffers.allocate(d.shape)
        print(f"[case] {case} form={fname}: good call", flush=True)
        assert _call(d, buf, form) == B.OK
        torch.cuda.synchronize()
        assert B.moe_workspace_status(buf.workspace, check=False) == B.OK
        G.check_against_oracle(li, buf, ref, tag=f"{case}/{fname}/before", rms_over_nonzero_rows=True)

        print(f"[case] {case} form={fname}: every wait runs out after 8 polls", flush=True)
        B.moe_workspace_wait_test(buf.workspace, 8, 1)
        buf.out.zero_()
        assert _call(d, buf, form) == B.OK          # the launches themselves succeed
        torch.cuda.synchronize()                    # ... and every kernel ends
        assert int(buf.miss_count.cpu()[0]) == -1, (case, fname, "miss_count must say that the call failed")
        assert bool(torch.isnan(buf.out).all()), (case, fname, "out must be NaN after a wait ran out")
        assert B.moe_workspace_status(buf.workspace, check=False) == B.ERR_LAUNCH
        assert "bounded wait" in B.moe_status_string(B.ERR_LAUNCH)
        assert B.moe_workspace_status(buf.workspace, check=False) == B.OK   # reported once, then cleared

        print(f"[case] {case} form={fname}: the same workspace again", flush=True)
        B.moe_workspace_wait_test(buf.workspace, 0, 0)
        for _ in range(2):
            buf.out.zero_()
            assert _call(d, buf, form) == B.OK
            torch.cuda.synchronize()
            assert B.moe_workspace_status(buf.workspace, check=False) == B.OK
            G.check_against_oracle(li, buf, ref, tag=f"{case}/{fname}/after", rms_over_nonzero_rows=True)


def test_a_workspace_that_served_another_shape_is_reported():
    """A workspace serves one layout between two moe_workspace_init calls: the first kernel of a call with
    another layout says so in the control block, the call marks its results, moe_workspace_status returns
    MOE_ERR_WORKSPACE, and after a new initialisation the other shape is served."""
    import gpu_util as G
    li_a = synth.make_layer(synth.small_recipe("ws_a", 4721, T=6, H=256, E=16, k=4, F=128, C=12, n_shared=1, F_shared=128))
    li_b = synth.make_layer(synth.small_recipe("ws_b", 4722, T=3, H=256, E=16, k=4, F=128, C=12, n_shared=1, F_shared=128))
    d_a, d_b = G.upload(li_a), G.upload(li_b)
    buf_a = B.LayerBuffers.allocate(d_a.shape)
    for form in (B.LAUNCH_THREE, B.LAUNCH_TWO, B.LAUNCH_ONE):
        B.moe_workspace_init(buf_a.workspace)
        assert _call(d_a, buf_a, form) == B.OK
        torch.cuda.synchronize()
        assert B.moe_workspace_status(buf_a.workspace, check=False) == B.OK
        G.check_against_oracle(li_a, buf_a, tag="shape A")
        # the smaller shape on the same (large enough) workspace, without a new initialisation
        buf_b = B.LayerBuffers.allocate(d_b.shape)
        buf_b.workspace = buf_a.workspace
        assert _call(d_b, buf_b, form) == B.OK
        torch.cuda.synchronize()
        assert int(buf_b.miss_count.cpu()[0]) == -1, form
        assert bool(torch.isnan(buf_b.out).all()), form
        assert B.moe_workspace_status(buf_a.workspace, check=False) == B.ERR_WORKSPACE
        B.moe_workspace_init(buf_a.workspace)
        assert _call(d_b, buf_b, form) == B.OK
        torch.cuda.synchronize()
        assert B.moe_workspace_status(buf_a.workspace, check=False) == B.OK
        G.check_against_oracle(li_b, buf_b, tag="shape B after a new initialisation")
