"""Helpers for the GPU parity tests: upload a synth.LayerInputs bundle, run the
HIP path through the C-ABI binding, and compare with the CPU oracle."""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

import oracle
from paper_2603_09983_amd import binding as B
from paper_2603_09983_amd import synth

RTOL_RMS = 2e-2      # FFN output: max |err| <= 2e-2 * RMS(oracle output)
GATE_ATOL = 1e-5     # gate weights
GATE_SUM_ATOL = 1e-6


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@dataclass
class DeviceLayer:
    shape: B.MoeShape
    hidden: torch.Tensor
    router_w: torch.Tensor
    router_bias: torch.Tensor | None
    slot_table: torch.Tensor
    w_gate: torch.Tensor | None
    w_up: torch.Tensor | None
    w_down: torch.Tensor | None
    sh_gate: torch.Tensor | None
    sh_up: torch.Tensor | None
    sh_down: torch.Tensor | None


def upload(li: synth.LayerInputs) -> DeviceLayer:
    s = li.shape
    pg, pu, pd = li.pools()
    has_pool = s.C > 0
    return DeviceLayer(
        B.make_shape(s.T, s.H, s.E, s.k, s.F, s.C, s.n_shared, s.F_shared),
        dev_bf16(li.hidden), dev(li.router_w), None if li.router_bias is None else dev(li.router_bias),
        dev(li.slot_table),
        dev_bf16(pg) if has_pool else None, dev_bf16(pu) if has_pool else None,
        dev_bf16(pd) if has_pool else None,
        None if li.sh_gate is None else dev_bf16(li.sh_gate),
        None if li.sh_up is None else dev_bf16(li.sh_up),
        None if li.sh_down is None else dev_bf16(li.sh_down))


def run_layer(d: DeviceLayer, buf: B.LayerBuffers | None = None, out_bf16=False, accumulate=False,
              form: int = B.LAUNCH_AUTO):
    """One moe_verify_layer call in the given launch form (a fresh workspace unless `buf` is given)."""
    buf = buf or B.LayerBuffers.allocate(d.shape, out_bf16=out_bf16)
    B.moe_verify_layer(B.with_form(d.shape, form), d.hidden, d.router_w, d.router_bias, d.slot_table, d.w_gate, d.w_up, d.w_down,
                       d.sh_gate, d.sh_up, d.sh_down, buf.topk_idx, buf.topk_w, buf.hist, buf.slot_idx,
                       buf.miss_list, buf.miss_count, buf.out, out_bf16, accumulate, buf.workspace)
    torch.cuda.synchronize()
    B.moe_workspace_status(buf.workspace)   # raises if a bounded wait inside a kernel ran out
    return buf


def rms(y: np.ndarray) -> float:
    return float(np.sqrt(np.mean(np.square(y, dtype=np.float64))))


def check_against_oracle(li: synth.LayerInputs, buf: B.LayerBuffers, ref: oracle.LayerResult | None = None,
                         tag: str = "", rms_over_nonzero_rows: bool = False):
    """Integer outputs bit-exact; gates within 1e-5; output within 2e-2 x RMS of the oracle output
    (rms_over_nonzero_rows: RMS over the token rows that receive anything; for layers where most
    tokens hit no resident expert the all-rows RMS is diluted by exact zeros)."""
    ref = ref or oracle.layer_from_inputs(li)
    idx = buf.topk_idx.cpu().numpy()
    assert np.array_equal(idx, ref.topk_idx), f"{tag} topk_idx"
    w = buf.topk_w.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(w - ref.gate)) <= GATE_ATOL, f"{tag} gate err {np.max(np.abs(w - ref.gate))}"
    assert np.max(np.abs(w.sum(axis=1) - 1.0)) <= GATE_SUM_ATOL, f"{tag} gate sum"
    assert np.array_equal(buf.hist.cpu().numpy(), ref.hist), f"{tag} hist"
    assert np.array_equal(buf.slot_idx.cpu().numpy(), ref.slot_idx), f"{tag} slot_idx"
    n = int(buf.miss_count.cpu().numpy()[0])
    assert n == ref.miss_count, f"{tag} miss_count {n} != {ref.miss_count}"
    assert np.array_equal(buf.miss_list.cpu().numpy()[:n], ref.miss_list), f"{tag} miss_list"
    y = buf.out.float().cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(y)), f"{tag} non-finite output"
    r = rms(ref.y)
    if rms_over_nonzero_rows and r > 0.0:
        rows = np.any(ref.y != 0.0, axis=1)
        assert np.all(y[~rows] == 0.0), f"{tag} a token without resident expert must get exact zeros"
        r = rms(ref.y[rows])
    err = float(np.max(np.abs(y - ref.y)))
    if r == 0.0:
        assert err == 0.0, f"{tag} expected exact zeros"
    else:
        assert err <= RTOL_RMS * r, f"{tag} max|err| {err:.3e} > {RTOL_RMS} * rms {r:.3e}"
    return err / r if r > 0 else 0.0
