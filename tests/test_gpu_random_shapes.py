"""Seeded random shapes through moe_verify_layer against the oracle: the corners between the kernel
variants (one or several contraction panels, one or two token groups, extra token passes, shapes the
streaming kernels do not take, empty caches, E not a multiple of the wavefront, k = 1 and k = E)."""
import numpy as np
import pytest

from paper_2603_09983_amd import synth

pytestmark = pytest.mark.gpu


def _shapes():
    rng = np.random.default_rng(2026)
    out = []
    for i in range(36):
        T = int(rng.choice([1, 2, 5, 9, 16, 17, 24, 32, 33, 47]))
        E = int(rng.choice([2, 7, 8, 16, 60, 64, 65, 130]))
        k = int(min(E, rng.choice([1, 2, 4, 6, 8])))
        if i % 9 == 0:
            k = E if E <= 8 else k
        H = int(rng.choice([64, 128, 256, 2048 + 64, 4096] if i % 4 == 0 else [64, 128, 192, 256, 320]))
        F = int(rng.choice([64, 128, 192, 2048 + 128] if i % 5 == 0 else [64, 128, 192, 256]))
        if i % 7 == 3:
            H, F = int(rng.choice([96, 160, 224])), int(rng.choice([96, 160]))   # not multiples of 64: general kernel
        C = int(rng.integers(0, E + 1))
        n_sh = int(rng.choice([0, 0, 1, 2]))
        Fs = int(rng.choice([64, 128, 192])) if n_sh else 0
        if H * F > 4096 * 256:   # keep the oracle quick
            F = 64
        out.append(dict(T=T, H=H, E=E, k=k, F=F, C=C, n_shared=n_sh, F_shared=Fs))
    return out


SHAPES = _shapes()


@pytest.mark.parametrize("i", range(len(SHAPES)))
def test_random_shape(i):
    import gpu_util as G
    kw = dict(SHAPES[i])
    hidden = "unit" if kw["E"] > 32 else "n002"
    li = synth.make_layer(synth.small_recipe(f"rand{i}", 9000 + i, hidden=hidden, **kw))
    print(f"[case] {i} {kw}", flush=True)
    buf = G.run_layer(G.upload(li))
    G.check_against_oracle(li, buf, tag=f"rand{i} {kw}", rms_over_nonzero_rows=True)
    if i % 3 == 0:   # bf16 output and accumulation on top of a previous result
        buf2 = G.run_layer(G.upload(li), out_bf16=True)
        ref = G.oracle.layer_from_inputs(li)
        y = buf2.out.float().cpu().numpy().astype(np.float64)
        rows = np.any(ref.y != 0.0, axis=1)
        if rows.any():   # bf16 rounding of the output adds up to 2^-9 of the largest element
            assert np.max(np.abs(y - ref.y)) <= G.RTOL_RMS * G.rms(ref.y[rows]) + 2.0 ** -8 * np.max(np.abs(ref.y))
