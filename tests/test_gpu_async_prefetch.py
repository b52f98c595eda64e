"""The combination the method exists for (Sec. 3.4, asynchronous prefetch): the cache manager's copy
(moe_pool_load) runs on a second stream while verify steps (moe_verify_layer) run on the first.  The copy fills
slots of ANOTHER layer's pool from an expert store (device memory; pinned host memory the device reads directly),
as the prefetch for layer l+1 does while layer l computes.  Checked: every verify step that ran beside the copy is
right, the layer whose experts were copied is right afterwards, no bounded wait inside a kernel ran out, and the
two really overlapped in time (events on both streams)."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2603_09983_amd import binding as B
from paper_2603_09983_amd import synth

pytestmark = pytest.mark.gpu


def _verify(d, buf, out, stream=None):
    B.moe_verify_layer(d.shape, d.hidden, d.router_w, d.router_bias, d.slot_table, d.w_gate, d.w_up, d.w_down,
                       d.sh_gate, d.sh_up, d.sh_down, buf.topk_idx, buf.topk_w, buf.hist, buf.slot_idx,
                       buf.miss_list, buf.miss_count, out, False, False, buf.workspace, stream=stream)


@pytest.mark.parametrize("where", ["device", "pinned_host"])
def test_verify_steps_beside_the_cache_managers_copy(where):
    import gpu_util as G
    base = synth.RECIPES["cfg2"]
    li_a = synth.make_layer(base, experts="resident")
    li_b = synth.make_layer(dataclasses.replace(base, seed=base.seed + 1000), experts="resident")
    s = li_a.shape
    d_a, d_b = G.upload(li_a), G.upload(li_b)
    ref_a, ref_b = oracle.layer_from_inputs(li_a), oracle.layer_from_inputs(li_b)

    # four experts of layer B that this batch uses "arrive": their slots hold zeros until the copy has run
    used = [e for e in np.flatnonzero(ref_b.hist > 0) if li_b.slot_table[e] >= 0][:4]
    assert len(used) == 4
    slots = [int(li_b.slot_table[e]) for e in used]
    store_idx = [1, 3, 4, 6]                      # where the store keeps them (a store with other entries between)
    host = [np.zeros((8, *w.shape[1:]), dtype=np.uint16) for w in (li_b.w_gate, li_b.w_up, li_b.w_down)]
    for i, e in zip(store_idx, used):
        for h, w in zip(host, (li_b.w_gate, li_b.w_up, li_b.w_down)):
            h[i] = w[e]
    if where == "device":
        store = [G.dev_bf16(h) for h in host]
    else:
        store = [torch.from_numpy(h.view(np.int16)).pin_memory() for h in host]   # allocated pinned, not registered
    for w in (d_b.w_gate, d_b.w_up, d_b.w_down):
        w[slots] = 0
    i32 = dict(dtype=torch.int32, device="cuda")
    fetch_list, fetch_slot = torch.tensor(store_idx, **i32), torch.tensor(slots, **i32)
    n_fetch = torch.tensor([4], **i32)

    buf_a, buf_b = B.LayerBuffers.allocate(d_a.shape), B.LayerBuffers.allocate(d_b.shape)
    _verify(d_b, buf_b, buf_b.out)
    torch.cuda.synchronize()
    y = buf_b.out.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(y - ref_b.y)) > G.RTOL_RMS * G.rms(ref_b.y), "the zeroed slots must matter"

    n_steps = 48
    loads = range(n_steps) if where == "device" else (0,)     # from the host one copy spans many verify steps
    outs = [torch.full_like(buf_a.out, float("nan")) for _ in range(n_steps)]
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()     # (both at the default priority)
    ev = {k: torch.cuda.Event(enable_timing=True) for k in ("load0", "load1", "step0", "step1")}
    torch.cuda.synchronize()
    print(f"[case] store in {where} memory: {len(loads)} copies beside {n_steps} verify steps", flush=True)
    ev["load0"].record(side)
    ev["step0"].record(main)
    for i in range(n_steps):
        if i in loads:
            B.moe_pool_load(*store, d_b.w_gate, d_b.w_up, d_b.w_down, fetch_list, fetch_slot, n_fetch, 4, s.H, s.F,
                            stream=side)
        _verify(d_a, buf_a, outs[i])
    ev["load1"].record(side)
    ev["step1"].record(main)
    main.wait_event(ev["load1"])                 # layer B's verify step needs the arrived experts
    _verify(d_b, buf_b, buf_b.out)
    torch.cuda.synchronize()

    assert B.moe_workspace_status(buf_a.workspace, check=False) == B.OK
    assert B.moe_workspace_status(buf_b.workspace, check=False) == B.OK
    # the two streams' work intersected in time
    assert ev["load0"].elapsed_time(ev["step1"]) > 0 and ev["step0"].elapsed_time(ev["load1"]) > 0
    print(f"[done] copies {ev['load0'].elapsed_time(ev['load1']) * 1e3:.0f} us, verify steps "
          f"{ev['step0'].elapsed_time(ev['step1']) * 1e3:.0f} us", flush=True)
    tol = G.RTOL_RMS * G.rms(ref_a.y)
    for i, o in enumerate(outs):
        err = float(np.max(np.abs(o.cpu().numpy().astype(np.float64) - ref_a.y)))
        assert err <= tol, (where, i, err, tol)
    G.check_against_oracle(li_a, dataclasses.replace(buf_a, out=outs[-1]), ref_a, tag=f"{where}/A")
    G.check_against_oracle(li_b, buf_b, ref_b, tag=f"{where}/B after the copy")
    pg = d_b.w_gate.view(torch.int16).cpu().numpy().view(np.uint16)
    for e, c in zip(used, slots):
        assert np.array_equal(pg[c], li_b.w_gate[e])
