"""Seeded random shapes in EVERY launch form the shape allows, each twice on one workspace, against the oracle.
Wider than test_gpu_random_shapes.py (sizes that are multiples of 8 only, hidden sizes whose panels are thirds,
up to three shared experts, empty and full caches), cheaper per case (small matrices), and the place where a rule
of the kernels' geometry that only some sizes break shows up: the panel-width rule for H = 2112 was found here."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_09983_amd import binding as B
from paper_2603_09983_amd import synth

pytestmark = pytest.mark.gpu

FORMS = {"auto": B.LAUNCH_AUTO, "three": B.LAUNCH_THREE, "two": B.LAUNCH_TWO, "one": B.LAUNCH_ONE,
         "route+one": B.LAUNCH_ROUTE_PLUS_ONE}


def _shape(rng):
    T = int(rng.choice([1, 2, 3, 5, 9, 15, 16, 17, 24, 31, 32, 33, 40, 64]))
    E = int(rng.choice([2, 7, 8, 16, 60, 64, 65, 128, 130]))
    k = int(min(E, rng.choice([1, 2, 4, 6, 8])))
    H = int(rng.choice([64, 128, 192, 256, 320, 512, 2048 + 64, 8 * int(rng.integers(8, 40))]))
    F = int(rng.choice([64, 128, 192, 256, 8 * int(rng.integers(8, 40)), 2048 + 128]))
    if H * F > 2112 * 256:   # keep the oracle quick
        F = 64
    C = int(rng.integers(0, E + 1))
    n_sh = int(rng.choice([0, 0, 1, 2, 3]))
    Fs = int(rng.choice([64, 128, 192, 8 * int(rng.integers(8, 30))])) if n_sh else 0
    return dict(T=T, H=H, E=E, k=k, F=F, C=C, n_shared=n_sh, F_shared=Fs)


@pytest.mark.parametrize("seed", [777, 1, 2])
def test_random_shapes_in_every_launch_form(seed):
    import gpu_util as G
    rng = np.random.default_rng(seed)
    ran = {f: 0 for f in FORMS}
    for i in range(60):
        kw = _shape(rng)
        li = synth.make_layer(synth.small_recipe(f"rf{seed}_{i}", 31000 + 1000 * (seed % 7) + i,
                                                 hidden="unit" if kw["E"] > 32 else "n002", **kw))
        d = G.upload(li)
        ref = oracle.layer_from_inputs(li)
        print(f"[case] seed {seed} #{i} {kw}", flush=True)
        for fname, form in FORMS.items():
            buf = B.LayerBuffers.allocate(d.shape)
            for again in (False, True):     # the second call: the same workspace, the call number moved on
                rc = B.moe_verify_layer(B.with_form(d.shape, form), d.hidden, d.router_w, d.router_bias, d.slot_table,
                                        d.w_gate, d.w_up, d.w_down, d.sh_gate, d.sh_up, d.sh_down, buf.topk_idx,
                                        buf.topk_w, buf.hist, buf.slot_idx, buf.miss_list, buf.miss_count, buf.out,
                                        False, False, buf.workspace, check=False)
                if rc == B.ERR_SHAPE and fname not in ("auto", "three"):
                    break                   # this shape does not allow this form
                assert rc == B.OK, (kw, fname, rc)
                torch.cuda.synchronize()
                assert B.moe_workspace_status(buf.workspace, check=False) == B.OK, (kw, fname)
                G.check_against_oracle(li, buf, ref, tag=f"seed {seed} #{i} {kw} {fname}", rms_over_nonzero_rows=True)
                ran[fname] += again
    assert ran["auto"] == 60 and ran["three"] == 60 and min(ran.values()) >= 10, ran
