"""Every launch form of moe_verify_layer against the oracle: three launches, two (routing inside the gate/up
kernel), one (routing, gate/up, down and the final sum in one kernel) and routing kernel + one-launch FFN.
Same outputs to the same bar in every form, at the named workloads' full sizes and at the corners of the
one-launch kernel and of the two-launch form (one token, sixteen tokens, 17-32 tokens, no shared expert, several shared experts, several contraction
panels, empty cache share, bf16 output, accumulation, repeated calls on one workspace)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_09983_amd import binding as B
from paper_2603_09983_amd import synth

pytestmark = pytest.mark.gpu

FORMS = {"three": B.LAUNCH_THREE, "two": B.LAUNCH_TWO, "one": B.LAUNCH_ONE, "route+one": B.LAUNCH_ROUTE_PLUS_ONE}


def _case(name):
    if name in synth.RECIPES:
        return synth.make_layer(synth.RECIPES[name], experts="resident")
    if name.startswith("sweep"):
        T, layer = (int(x) for x in name[5:].split("_"))
        return synth.make_layer(synth.sweep_recipe(T, layer), hidden_seed=synth.sweep_hidden_seed(T), experts="resident")
    kw = {
        "one_token": dict(T=1, H=256, E=16, k=4, F=192, C=9),
        "sixteen_tokens": dict(T=16, H=512, E=64, k=6, F=384, C=40, n_shared=1, F_shared=128, hidden="unit"),
        "three_shared": dict(T=7, H=256, E=8, k=2, F=128, C=5, n_shared=3, F_shared=192),
        "panels": dict(T=4, H=4096, E=8, k=2, F=64, C=6, n_shared=1, F_shared=2048 + 128),
        "wide_shared_down": dict(T=5, H=128, E=8, k=3, F=128, C=8, n_shared=1, F_shared=4096 + 256),
        "all_miss": dict(T=6, H=128, E=16, k=2, F=64, C=1, n_shared=1, F_shared=64),
        "k_equals_e": dict(T=3, H=64, E=4, k=4, F=64, C=4),
        "e128": dict(T=9, H=256, E=128, k=8, F=128, C=64, hidden="unit"),
        # 17-32 tokens: two token groups per pass; the two-launch form ranks two tokens per wavefront
        "twenty_four": dict(T=24, H=512, E=64, k=6, F=384, C=40, n_shared=1, F_shared=128, hidden="unit"),
        "thirty_two_e128": dict(T=32, H=256, E=128, k=8, F=128, C=96, hidden="unit"),
        "panels_of_2112": dict(T=5, H=2112, E=7, k=2, F=256, C=3, n_shared=3, F_shared=192),
    }[name]
    return synth.make_layer(synth.small_recipe(name, 8800 + len(name), **kw))


CASES = ["cfg1", "cfg2", "cfg3", "cfg4_c4", "sweep1_11", "sweep5_0", "sweep9_23", "sweep17_11", "one_token",
         "sixteen_tokens", "three_shared", "panels", "wide_shared_down", "all_miss", "k_equals_e", "e128", "twenty_four",
         "thirty_two_e128", "panels_of_2112"]


@pytest.mark.parametrize("case", CASES)
def test_launch_forms_agree_with_the_oracle(case):
    import gpu_util as G
    li = _case(case)
    d = G.upload(li)
    ref = oracle.layer_from_inputs(li)
    ran = []
    for fname, form in FORMS.items():
        buf = B.LayerBuffers.allocate(d.shape)
        rc = B.moe_verify_layer(B.with_form(d.shape, form), d.hidden, d.router_w, d.router_bias, d.slot_table, d.w_gate,
                                d.w_up, d.w_down, d.sh_gate, d.sh_up, d.sh_down, buf.topk_idx, buf.topk_w, buf.hist,
                                buf.slot_idx, buf.miss_list, buf.miss_count, buf.out, False, False, buf.workspace,
                                check=False)
        if rc == B.ERR_SHAPE:
            continue                      # this shape does not allow this form
        assert rc == B.OK, (case, fname, rc)
        print(f"[case] {case} form={fname} shape={li.shape}", flush=True)
        torch.cuda.synchronize()
        B.moe_workspace_status(buf.workspace)
        G.check_against_oracle(li, buf, ref, tag=f"{case}/{fname}", rms_over_nonzero_rows=True)
        # the same workspace again (the call number moves on), bf16 output on top of a previous result
        half = torch.full_like(buf.out, 0.5).to(torch.bfloat16)
        B.moe_verify_layer(B.with_form(d.shape, form), d.hidden, d.router_w, d.router_bias, d.slot_table, d.w_gate,
                           d.w_up, d.w_down, d.sh_gate, d.sh_up, d.sh_down, buf.topk_idx, buf.topk_w, buf.hist,
                           buf.slot_idx, buf.miss_list, buf.miss_count, half, True, True, buf.workspace)
        torch.cuda.synchronize()
        B.moe_workspace_status(buf.workspace)
        y = half.float().cpu().numpy().astype(np.float64)
        want = ref.y + 0.5
        tol = G.RTOL_RMS * max(G.rms(ref.y), 1e-30) + 2.0 ** -8 * np.max(np.abs(want))   # + bf16 rounding of the sum
        assert np.max(np.abs(y - want)) <= tol, (case, fname, "bf16 accumulate")
        ran.append(fname)
    assert "three" in ran
    if li.shape.T <= 32 and li.shape.E <= 128 and li.shape.C >= 1 and li.shape.H % 64 == 0 and li.shape.F % 64 == 0:
        assert "two" in ran, (case, ran)
    if li.shape.T <= 16 and li.shape.E <= 128 and li.shape.C >= 1 and li.shape.H % 64 == 0 and li.shape.F % 64 == 0:
        assert "one" in ran and "route+one" in ran, (case, ran)
