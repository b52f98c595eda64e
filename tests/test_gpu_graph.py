"""The layer call inside a captured HIP graph: every entry point only enqueues kernels on the given
stream (no allocation, no memset, no synchronisation), so a launch-bound sequence of layers can be
replayed from a graph.  Replays are interleaved with eager work and synchronisations and each one
is compared with the eager result (bit-exact: the kernels are deterministic)."""
import numpy as np
import pytest
import torch

from paper_2603_09983_amd import synth

pytestmark = pytest.mark.gpu


def test_verify_layer_replays_from_a_graph():
    from paper_2603_09983_amd import binding as B
    import gpu_util as G
    recs = [synth.small_recipe(f"graph{i}", 40 + i, T=9, H=256, E=64, k=6, F=256, C=32, n_shared=1, F_shared=128)
            for i in range(2)]
    layers = [synth.make_layer(r) for r in recs]
    devs = [G.upload(li) for li in layers]
    eager = []
    for d in devs:
        buf = G.run_layer(d)
        eager.append({k: getattr(buf, k).clone() for k in ("topk_idx", "topk_w", "hist", "slot_idx", "miss_count", "out")})
    bufs = [B.LayerBuffers.allocate(d.shape) for d in devs]

    def call(d, buf):
        B.moe_verify_layer(d.shape, d.hidden, d.router_w, d.router_bias, d.slot_table, d.w_gate, d.w_up, d.w_down,
                           d.sh_gate, d.sh_up, d.sh_down, buf.topk_idx, buf.topk_w, buf.hist, buf.slot_idx,
                           buf.miss_list, buf.miss_count, buf.out, False, False, buf.workspace)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # warm-up on the capture stream (first-launch set-up must not be captured)
        for d, buf in zip(devs, bufs):
            call(d, buf)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for d, buf in zip(devs, bufs):     # two layers back to back in one graph
            call(d, buf)
    scratch = torch.zeros(1 << 20, device="cuda")
    for replay in range(4):
        for buf in bufs:
            buf.out.fill_(float("nan"))
            buf.topk_idx.fill_(-1)
        scratch.add_(1.0).sum().item()     # eager work and a synchronisation between replays
        graph.replay()
        torch.cuda.synchronize()
        for i, buf in enumerate(bufs):
            B.moe_workspace_status(buf.workspace)
            for k, want in eager[i].items():
                assert torch.equal(getattr(buf, k), want), f"replay {replay} layer {i}: {k}"
        # an eager call on the same buffers between replays must not disturb the next replay
        call(devs[0], bufs[0])
        torch.cuda.synchronize()
