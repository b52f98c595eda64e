#!/usr/bin/env python3
"""Benchmark of the verify-step MoE layer on one MI355X.

A step = one pass of the whole hot path (moe_verify_layer: routing, histogram,
slot resolve, grouped SwiGLU FFN, combine) over one verification batch.  The
default workload is the small-MoE verify step (T=9, H=2048, 64 experts, top-6,
2 shared experts, cache capacity 32).  Consecutive steps run DIFFERENT layers
(independent seeded weights, router and hidden states), rotating over enough
weight copies that the streamed bytes exceed the 256 MB last-level cache many
times over, so every step reads its expert weights from HBM.

Prints ONE JSON line: whole-job expert-weight GB/s (value), ms per step, the
HBM roofline of the dominant kernel measured with HIP events inside this run,
the same whole-layer measurement for the other two small-batch workloads of
the 64-expert class (`north_star_rows`), every launch form of the layer, and
the CPU oracle timed on this machine's host cores (a reported baseline only).

Timers: `value`, `ms_per_step`, `whole_layer_frac`, `north_star_rows` and
`launch_forms` are host wall clock between two device synchronisations around
K back-to-back steps; `roofline.achieved` is HIP-event pairs around every
launch of the dominant kernel (uncorrected: an empty event pair itself spans a
few microseconds, reported as `event_pair_overhead_us`); `roofline.frac_rocprof`
and `roofline.traffic` are read from the recorded rocprofv3 summary under
profiles/ and are null when that summary is of another kernel or other sources.

After every timed region the workspace's control block is read back
(moe_workspace_status): a run in which a bounded wait inside a kernel ran out
is not a measurement, and the program stops instead of printing it.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# rocprofv3 figures of the dominant kernel of the default workload (average duration from --kernel-trace
# --stats; FETCH_SIZE and WRITE_SIZE from two --pmc runs with their calibration factor), as `key = value`
# lines, with the name of the kernel and a hash of the kernel sources they were recorded for
RECORDED = os.path.join(ROOT, "profiles", "recorded_counters_cfg2.txt")
KERNEL_SOURCES = ("stream.hip", "route_device.h", "route.hip", "moe_internal.h")


def sources_hash() -> str:
    import hashlib
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2603_09983_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def recorded_counters(workload: str, kernel: str):
    """(dict, why-not): the recorded rocprofv3 figures when they are of this workload, this kernel and these sources."""
    if workload != "cfg2" or not os.path.exists(RECORDED):
        return None, "no rocprofv3 summary recorded for this workload"
    rec = {}
    with open(RECORDED) as fh:
        for line in fh:
            if "=" in line and not line.lstrip().startswith("#"):
                k, v = line.split("=", 1)
                rec[k.strip()] = v.strip()
    if rec.get("kernel") != kernel:
        return None, f"recorded for another kernel ({rec.get('kernel')})"
    if rec.get("sources_sha256_16") != sources_hash():
        return None, "recorded for other kernel sources than the ones in this tree"
    return rec, None


def parse_args():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=240)
    p.add_argument("--warmup", type=int, default=48)
    p.add_argument("--workload", default="cfg2",
                   help="cfg2 | cfg3 | cfg4_c8 | cfg4_c4 | cfg5_T<n> (24-layer sweep at T=n)")
    p.add_argument("--copies", type=int, default=0, help="distinct layers to rotate over (0 = auto)")
    p.add_argument("--form", default="auto", choices=["auto", "three", "two", "one", "route+one"],
                   help="launch form of moe_verify_layer (moe_shape_t::launch_form)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-estimator", action="store_true", help="skip the utility-estimator measurement")
    p.add_argument("--no-forms", action="store_true",
                   help="skip the extra timed regions that run the same steps in every other launch form")
    p.add_argument("--no-rows", action="store_true",
                   help="skip the whole-layer measurement of the other small-batch workloads (cfg5 T=5 and T=9)")
    p.add_argument("--graph", action="store_true",
                   help="timed region 1 replays a captured HIP graph of one pass over the layers (lifts the "
                        "host's launch rate off small layers); steps must be a multiple of the layer count")
    p.add_argument("--cpu-seconds", type=float, default=10.0)
    p.add_argument("--no-prefetch-overlap", action="store_true",
                   help="skip the verify steps with the cache manager's copy running beside them on a second "
                        "stream (store in device memory, then in pinned host memory)")
    p.add_argument("--profile-run", action="store_true",
                   help="the run a profiler is attached to: the default workload in the default form only "
                        "(no other forms, workloads, estimator, overlap or CPU baseline)")
    p.add_argument("--timeline", action="store_true",
                   help="with a library built with the timeline stamps (build.py --trace, MOE_SPAC_LIB): print to "
                        "stderr when the workgroups of the two streaming kernels reach each point of their life")
    p.add_argument("--calibration-copy", action="store_true",
                   help="also run one plain 1 GiB device copy (a kernel of known traffic, for scaling "
                        "rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    return p.parse_args()


def build_layers(workload: str, copies: int):
    """List of synth.LayerInputs (resident experts only) for the chosen workload."""
    import dataclasses
    from paper_2603_09983_amd import synth
    layers = []
    if workload.startswith("cfg5_T"):
        T = int(workload[len("cfg5_T"):])
        n = copies or synth.SWEEP_LAYERS
        for l in range(n):
            layers.append(synth.make_layer(synth.sweep_recipe(T, l), hidden_seed=synth.sweep_hidden_seed(T),
                                           experts="resident"))
        desc = f"cfg5 sweep: T={T} H=2048 E=64 k=6 F=1408 C=48, {n} independent layers back to back"
    else:
        base = synth.RECIPES[workload]
        s = base.shape
        per_copy = s.C * 6 * s.H * s.F + s.n_shared * 6 * s.H * s.F_shared
        n = copies or max(2, min(16, int(6e9 // per_copy)))
        for i in range(n):
            layers.append(synth.make_layer(dataclasses.replace(base, seed=base.seed + 1000 * i),
                                           experts="resident"))
        desc = (f"{workload}: T={s.T} H={s.H} E={s.E} k={s.k} F={s.F} C={s.C} "
                f"shared={s.n_shared}x{s.F_shared}, rotating over {n} independent layers")
    return layers, desc


def print_timeline(B, torch, np, step, n_layers):
    """Per streaming kernel of three consecutive layer calls: min / median / max over the workgroups of the
    time (us after the first workgroup's start) at which they have the lists in LDS, have consumed their
    first tile, leave their loop, have stored their results and end; the loop-end mean per XCD."""
    for i in range(min(3, n_layers)):
        step(i)
        torch.cuda.synchronize()
        got = B.moe_profile_stream_timeline()
        words, lwords = got if got is not None else (None, None)
        if words is None:
            print("[timeline] the loaded library has no timeline stamps (python paper_2603_09983_amd/build.py "
                  "--trace; MOE_SPAC_LIB=paper_2603_09983_amd/libmoe_spac_trace.so)", file=sys.stderr)
            return
        tl = lwords.astype(np.int64)
        tl = tl[tl[:, 5] > 0]
        if len(tl) and tl[:, 0].min() > max(words[0][:, 0].max(), words[1][:, 0].max()):
            # the one-launch layer kernel ran last: start | lists | first tile | enters the down part | loop end | end
            us = (tl[:, :6] - tl[:, 0].min()) / 100.0
            us[:, 3] = np.where(tl[:, 3] > 0, us[:, 3], np.nan)

            def q(x):
                return "%5.1f/%5.1f/%5.1f" % (np.nanmin(x), np.nanmedian(x), np.nanmax(x))
            print(f"[timeline] layer {i} one launch ({len(tl)} workgroups, {(tl[:, 6] >> 32).min()}-{(tl[:, 6] >> 32).max()} gate/up and "
                  f"{(tl[:, 6] & 0xffffffff).min()}-{(tl[:, 6] & 0xffffffff).max()} down items each): start {q(us[:, 0])} | "
                  f"lists {q(us[:, 1])} | first tile {q(us[:, 2])} | down part {q(us[:, 3])} | loop end {q(us[:, 4])} | "
                  f"end {q(us[:, 5])}", file=sys.stderr)
            xcd = np.arange(len(tl)) % 8
            print("[timeline]     down part entered, mean per XCD: " +
                  " ".join("%.1f" % np.nanmean(us[xcd == x, 3]) for x in range(8)), file=sys.stderr)
            print("[timeline]     loop end, mean per XCD: " +
                  " ".join("%.1f" % us[xcd == x, 4].mean() for x in range(8)), file=sys.stderr)
            names = ("wait", "park", "store", "request", "barrier1", "multiply", "barrier2", "walk")
            steps = np.maximum(tl[:, 7] - 1, 1)
            for wv, off in ((0, 8), (15, 16)):
                cyc = tl[:, off:off + 8] / steps[:, None]
                print(f"[timeline]     wavefront {wv:2d}, shader cycles per step (median over workgroups): " +
                      " ".join(f"{nm} {np.median(cyc[:, j]):.0f}" for j, nm in enumerate(names)) +
                      f" | sum {np.median(cyc.sum(axis=1)):.0f}", file=sys.stderr)
            continue
        for ki, name in enumerate(("gate/up", "down")):
            t = words[ki].astype(np.int64)
            t = t[t[:, 5] > 0]
            if not len(t):
                continue
            us = (t[:, :6] - t[:, 0].min()) / 100.0

            def q(x):
                return "%5.1f/%5.1f/%5.1f" % (x.min(), np.median(x), x.max())
            print(f"[timeline] layer {i} {name:7s} ({len(t)} workgroups, {t[:, 6].min()}-{t[:, 6].max()} items each): "
                  f"start {q(us[:, 0])} | lists {q(us[:, 1])} | first tile {q(us[:, 2])} | loop end {q(us[:, 3])} | "
                  f"stored {q(us[:, 4])} | end {q(us[:, 5])}", file=sys.stderr)
            xcd = np.arange(len(t)) % 8
            print("[timeline]     loop end, mean per XCD: " +
                  " ".join("%.1f" % us[xcd == x, 3].mean() for x in range(8)), file=sys.stderr)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the verify-step MoE layer is a single-device kernel path; "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2603_09983_amd import binding as B
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import gpu_util as G

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    if args.profile_run:
        args.no_forms = args.no_rows = args.no_estimator = args.no_cpu_baseline = args.no_prefetch_overlap = True
    FORMS = {"auto": B.LAUNCH_AUTO, "three": B.LAUNCH_THREE, "two": B.LAUNCH_TWO, "one": B.LAUNCH_ONE,
             "route+one": B.LAUNCH_ROUTE_PLUS_ONE}

    def healthy(workspace, what):
        """Stops the program when a bounded wait inside a kernel ran out during the region just timed."""
        if B.moe_workspace_status(workspace, check=False) != B.OK:
            sys.exit(f"bench.py: {what}: {B.moe_status_string(B.ERR_LAUNCH)}; nothing of this run is a measurement")

    class Workload:
        """Uploaded layers of one workload, one set of output buffers, the algorithmic bytes of every layer."""

        def __init__(self, name, copies, keep_host_weights=True):
            t_gen = time.time()
            self.layers, self.desc = build_layers(name, copies)
            self.dev = []
            for li in self.layers:
                self.dev.append(G.upload(li))
                if not keep_host_weights:       # (tens of GB over a 24-layer sweep; only the device copy is used)
                    li.w_gate = li.w_up = li.w_down = None
            self.finish(time.time() - t_gen)

        def finish(self, secs):
            self.shape = self.layers[0].shape
            self.buf = B.LayerBuffers.allocate(self.dev[0].shape)
            print(f"[bench] {self.desc}; inputs built and uploaded in {secs:.1f}s", file=sys.stderr, flush=True)
            # algorithmic expert-weight bytes of each layer, from its actual routing (one untimed pass)
            sh = self.shape
            per_expert = 6 * sh.H * sh.F
            shared_bytes = sh.n_shared * 6 * sh.H * sh.F_shared
            self.layer_bytes = []
            for i, li in enumerate(self.layers):
                self.step(i, B.LAUNCH_AUTO)
                torch.cuda.synchronize()
                hist = self.buf.hist.cpu().numpy()
                u_res = int(((hist > 0) & (li.slot_table >= 0)).sum())
                self.layer_bytes.append(u_res * per_expert + shared_bytes)
            healthy(self.buf.workspace, "first pass")

        def with_tokens(self, T):
            """The same layers (weights, router, residency) under another batch size: new hidden states only."""
            import copy
            import dataclasses
            from paper_2603_09983_amd import synth
            t_gen = time.time()
            w = copy.copy(self)
            w.layers, w.dev = [], []
            for l, (li, d) in enumerate(zip(self.layers, self.dev)):
                r = synth.sweep_recipe(T, l)
                assert r.seed == li.recipe.seed
                hid = synth.hidden_states(synth.sweep_hidden_seed(T), T, r.shape.H, r.hidden, li.router_w, li.router_bias,
                                          r.shape.k, synth.MARGIN)
                w.layers.append(dataclasses.replace(li, recipe=r, shape=r.shape, hidden=hid))
                s0 = d.shape
                w.dev.append(dataclasses.replace(d, shape=B.make_shape(T, s0.H, s0.E, s0.k, s0.F, s0.C, s0.n_shared,
                                                                       s0.F_shared), hidden=G.dev_bf16(hid)))
            w.desc = self.desc.replace(f"T={self.shape.T} ", f"T={T} ")
            w.finish(time.time() - t_gen)
            return w

        def step(self, i, form):
            d, buf = self.dev[i % len(self.dev)], self.buf
            B.moe_verify_layer(B.with_form(d.shape, form), d.hidden, d.router_w, d.router_bias, d.slot_table, d.w_gate,
                               d.w_up, d.w_down, d.sh_gate, d.sh_up, d.sh_down, buf.topk_idx, buf.topk_w, buf.hist,
                               buf.slot_idx, buf.miss_list, buf.miss_count, buf.out, False, False, buf.workspace)

        def bytes_of(self, steps):
            return sum(self.layer_bytes[i % len(self.layers)] for i in range(steps))

        def timed(self, form, steps, warmup, what):
            """Seconds of `steps` back-to-back steps: host wall clock between two device synchronisations."""
            for i in range(warmup):
                self.step(i, form)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(steps):
                self.step(i, form)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            healthy(self.buf.workspace, what)
            return t1 - t0

        def chain(self, form, reps, warmup, what):
            """One pass over all layers of the workload, back to back, `reps` times, each pass between two HIP
            events on the launch stream: median, 10th and 90th percentile of the time per layer."""
            n = len(self.layers)
            for r in range(warmup):
                for i in range(n):
                    self.step(i, form)
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            torch.cuda.synchronize()
            for r in range(reps):
                ev[r][0].record()
                for i in range(n):
                    self.step(i, form)
                ev[r][1].record()
            torch.cuda.synchronize()
            healthy(self.buf.workspace, what)
            us = np.array([a.elapsed_time(b) for a, b in ev]) * 1e3 / n
            return {"passes": reps, "warmup_passes": warmup, "layers_per_pass": n,
                    "us_per_layer_median": round(float(np.median(us)), 2),
                    "us_per_layer_p10": round(float(np.percentile(us, 10)), 2),
                    "us_per_layer_p90": round(float(np.percentile(us, 90)), 2),
                    "timer": "one HIP-event pair around each pass"}

        def row(self, form, steps, warmup, what, chain_reps=0):
            secs = self.timed(form, steps, warmup, what)
            gbs = self.bytes_of(steps) / secs / 1e9
            out = {"us_per_layer": round(secs * 1e6 / steps, 2), "GBs": round(gbs, 1),
                   "whole_layer_frac": round(gbs / HBM_PEAK_GBS, 4),
                   "mean_weight_bytes_per_layer": int(np.mean(self.layer_bytes)), "steps": steps, "warmup": warmup}
            if chain_reps:
                out["chain"] = self.chain(form, chain_reps, 20, what + ", pass by pass")
            return out

    wl = Workload(args.workload, args.copies)
    layers, dev_layers, shape, buf, desc, layer_bytes = wl.layers, wl.dev, wl.shape, wl.buf, wl.desc, wl.layer_bytes
    form = FORMS[args.form]

    def step(i):
        wl.step(i, form)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # timed region 1: K steps, wall clock between synchronisations -> value
    if args.graph:
        if args.steps % len(layers):
            sys.exit(f"--graph: --steps must be a multiple of {len(layers)}")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for i in range(len(layers)):
                step(i)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps // len(layers)):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    else:
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    healthy(buf.workspace, "timed region 1")
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    bytes_total = wl.bytes_of(args.steps)
    gbs = bytes_total / (t1 - t0) / 1e9

    # timed region 2: the same K steps with HIP events around every kernel (on the launch stream); once untimed
    # first, so that the library has made its event pairs before the pass that counts
    for _ in range(2):
        B.moe_profile_enable(True)
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        B.moe_profile_enable(False)
    healthy(buf.workspace, "timed region 2")
    raw = {kind: B.moe_profile_read(kind) for kind in range(B.KERNEL_KINDS)}
    # An event pair with nothing between its two records still spans a few microseconds (the queue going
    # from one packet to the next).  That interval is measured here, live, and reported beside every
    # bracketed kernel's average; the roofline figure uses the uncorrected average.
    ev_us = B.moe_profile_event_overhead(512) * 1e3
    kernels = {}
    for kind, (ms, n) in raw.items():
        if n:
            kernels[B.moe_profile_kernel_name(kind)] = {"launches": n, "avg_us_event_pair": round(ms * 1e3 / n, 2),
                                                        "avg_us_minus_empty_pair": round(ms * 1e3 / n - ev_us, 2)}
    # dominant kernel: the one-launch layer kernel carries every expert-weight byte of the layer; in the
    # forms with two streaming launches it is the gate/up stream (2/3 of the bytes)
    layer_ms, layer_n = raw[B.KERNEL_LAYER]
    ffn_ms, ffn_n = raw[B.KERNEL_FFN]
    down_ms, down_n = raw[B.KERNEL_DOWN]
    if layer_n:
        dom_name, dom_ms, dom_n, share = "layer_kernel", layer_ms, layer_n, 1.0
        dom_what = "gate/up + down + final sum in one launch"
    else:
        dom_name = "stream_kernel<gate/up>" if down_n else "ffn_kernel"
        dom_what = ("gate/up stream" + (", routing steps at its head" if not raw[B.KERNEL_ROUTE][1] else "")) if down_n \
            else "gate/up/down fused"
        dom_ms, dom_n, share = ffn_ms, ffn_n, (2.0 / 3.0 if down_n else 1.0)
    dom_avg_s = dom_ms * 1e-3 / dom_n
    bytes_per_launch = share * bytes_total / args.steps
    achieved = bytes_per_launch / dom_avg_s / 1e9
    rec, why_not = recorded_counters(args.workload if not args.copies and args.form == "auto" else "", dom_name)
    roofline = {"bound": "hbm", "kernel": dom_name, "kernel_does": dom_what,
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "timer": "HIP event pairs around every launch, uncorrected",
                "avg_kernel_us": round(dom_avg_s * 1e6, 2), "event_pair_overhead_us": round(ev_us, 2),
                "frac_minus_empty_pair": round(bytes_per_launch / (dom_avg_s - ev_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                "algorithmic_bytes_per_launch": int(bytes_per_launch),
                "traffic": None, "frac_rocprof": None, "recorded": why_not, "kernels": kernels}
    if rec:
        roofline["traffic"] = int((float(rec["fetch_size_kib"]) * float(rec["fetch_scale"]) + float(rec["write_size_kib"])) * 1024)
        roofline["frac_rocprof"] = round(float(rec["algorithmic_bytes_per_launch"]) / float(rec["rocprof_avg_ns"]) / HBM_PEAK_GBS, 4)
        roofline["recorded"] = {"file": os.path.relpath(RECORDED, ROOT), "rocprof_avg_ns": float(rec["rocprof_avg_ns"]),
                                "note": "a recorded run of the same command, kernel and sources, not this run"}
    if down_n and not layer_n:
        d_s = down_ms * 1e-3 / down_n
        roofline["down_kernel"] = {"achieved": round((bytes_total / args.steps / 3.0) / d_s / 1e9, 1),
                                   "avg_kernel_us": round(d_s * 1e6, 2)}

    # every other launch form of the layer on the same steps, timed like region 1
    launch_forms = None
    if not args.no_forms and not args.graph:
        launch_forms = {"timer": "host wall clock between two device synchronisations"}
        for fname, f in FORMS.items():
            if fname == "auto":
                continue
            d0 = dev_layers[0]
            rc = B.moe_verify_layer(B.with_form(d0.shape, f), d0.hidden, d0.router_w, d0.router_bias, d0.slot_table,
                                    d0.w_gate, d0.w_up, d0.w_down, d0.sh_gate, d0.sh_up, d0.sh_down, buf.topk_idx,
                                    buf.topk_w, buf.hist, buf.slot_idx, buf.miss_list, buf.miss_count, buf.out, False,
                                    False, buf.workspace, check=False)
            if rc == B.ERR_SHAPE:
                continue            # this shape does not allow this form
            launch_forms[fname] = wl.row(f, args.steps, args.warmup, "launch form " + fname)

    # the other two small-batch workloads the 70 % target is stated for, each timed like region 1 in the default form
    rows = {args.workload: {"us_per_layer": round(ms_per_step * 1e3, 2), "GBs": round(gbs, 1),
                            "whole_layer_frac": round(gbs / HBM_PEAK_GBS, 4),
                            "mean_weight_bytes_per_layer": int(np.mean(layer_bytes)), "steps": args.steps,
                            "warmup": args.warmup}}
    if not args.no_rows and args.workload == "cfg2" and not args.graph:
        sweep = Workload("cfg5_T9", 0, keep_host_weights=False)
        rows[args.workload]["chain"] = wl.chain(form, 100, 20, "cfg2, pass by pass")
        rows["cfg5_T9"] = sweep.row(form, 240, 48, "cfg5 T=9", chain_reps=100)
        sweep5 = sweep.with_tokens(5)
        rows["cfg5_T5"] = sweep5.row(form, 240, 48, "cfg5 T=5", chain_reps=100)
        del sweep, sweep5
        torch.cuda.empty_cache()
    rows["timer"] = ("us_per_layer: host wall clock between two device synchronisations around the steps, inputs resident; "
                     "chain: HIP events around each pass over the workload's layers, 20 warm-up passes + 100 timed ones")

    # NEXT row: the Speculative Utility Estimator consuming the histograms of 24 layers per inference
    # step (one launch for all layers); frequencies are synthetic histograms of T*k assignments.
    est = None
    if not args.no_estimator:
        L_est, K_est, gamma = 24, 4, shape.T - 1
        rng = np.random.default_rng(0)
        fr = np.zeros((8, L_est, shape.E), dtype=np.int32)
        for t in range(8):
            for l in range(L_est):
                for _ in range(shape.T):
                    fr[t, l, rng.choice(shape.E, size=shape.k, replace=False)] += 1
        d_fr = torch.from_numpy(fr).cuda()
        i32 = dict(dtype=torch.int32, device="cuda")
        st = [torch.zeros((L_est, shape.E), **i32) for _ in range(4)]
        d_tab = torch.from_numpy(np.stack([layers[i % len(layers)].slot_table for i in range(L_est)])).cuda()
        d_n = torch.zeros((L_est, K_est + 1), **i32)
        B.moe_utility_init(*st, L_est, shape.E, gamma)
        for t in range(16):
            B.moe_utility_update(d_fr[t % 8], *st, d_tab, d_n, L_est, shape.E, K_est, 1, 10)
        torch.cuda.synchronize()
        # ... and the balancer's threshold per layer from those counts (tables r_c, r_g: synthetic, monotone)
        r_c = torch.from_numpy(np.sort(rng.random((L_est, K_est + 1)), axis=1)).cuda()
        r_g = torch.from_numpy(np.ascontiguousarray(np.sort(rng.random((L_est, K_est + 1)), axis=1)[:, ::-1])).cuda()
        bal_p = B.BalanceParams(40.0, 3.0, 6.0, 600.0, L_est, 6 * shape.H * shape.F, 16 * 6 * shape.H * shape.F)
        d_tau = torch.zeros(L_est, **i32)
        B.moe_balance_threshold(d_fr[0], d_n, r_c, r_g, L_est, shape.E, K_est, gamma, shape.k, bal_p, d_tau)
        torch.cuda.synchronize()
        B.moe_profile_enable(True)
        n_est = 200
        for t in range(n_est):
            B.moe_utility_update(d_fr[t % 8], *st, d_tab, d_n, L_est, shape.E, K_est, 1, 10)
            B.moe_balance_threshold(d_fr[t % 8], d_n, r_c, r_g, L_est, shape.E, K_est, gamma, shape.k, bal_p, d_tau)
        torch.cuda.synchronize()
        B.moe_profile_enable(False)
        ms, n = B.moe_profile_read(B.KERNEL_ESTIMATOR)
        bal_ms, bal_n = B.moe_profile_read(B.KERNEL_BALANCER)
        est_us = ms * 1e3 / n - ev_us
        est_bytes = L_est * shape.E * 4 * (6 + 4) + L_est * (K_est + 1) * 4   # 6 words read, 4 written per expert
        est = {"kernel": "utility_update_kernel", "layers": L_est, "experts": shape.E, "K": K_est,
               "lambda": "1/10", "avg_us": round(est_us, 2), "avg_us_event_pair": round(ms * 1e3 / n, 2),
               "bound": "latency", "algorithmic_bytes": est_bytes,
               "note": "one launch advances all layers by one inference step and counts n(tau)",
               "balancer": {"kernel": "balance_kernel", "avg_us": round(bal_ms * 1e3 / bal_n - ev_us, 2),
                            "avg_us_event_pair": round(bal_ms * 1e3 / bal_n, 2), "bound": "latency"}}
        # ... and the cache manager: one planning step for all layers, then the copy of 4 fetched experts
        # of one layer from a full expert store (device memory here) into pool slots
        if shape.C >= 4:
            d_ev = torch.zeros((L_est, shape.E), **i32)
            d_fl, d_fs = torch.zeros((L_est, shape.C), **i32), torch.zeros((L_est, shape.C), **i32)
            d_ne, d_nf = torch.zeros(L_est, **i32), torch.zeros(L_est, **i32)
            tab0 = d_tab.clone()
            n_plan = 100
            B.moe_profile_enable(True)
            for t in range(n_plan):
                d_tab.copy_(tab0)
                B.moe_cache_plan(st[1], None, d_tab, d_tau, None, L_est, shape.E, shape.C, K_est, d_ev, d_ne, d_fl,
                                 d_fs, d_nf)
            torch.cuda.synchronize()
            B.moe_profile_enable(False)
            plan_ms, plan_n = B.moe_profile_read(B.KERNEL_CACHE_PLAN)
            n_move = 4
            store = [torch.empty((n_move * 3, *w.shape[1:]), dtype=w.dtype, device="cuda").normal_()
                     for w in (dev_layers[0].w_gate, dev_layers[0].w_up, dev_layers[0].w_down)]
            mv_list = torch.arange(0, n_move * 3, 3, **i32)
            mv_slot = torch.arange(n_move, **i32)
            mv_n = torch.full((1,), n_move, **i32)
            d0 = dev_layers[0]
            saved = [w[:n_move].clone() for w in (d0.w_gate, d0.w_up, d0.w_down)]
            B.moe_pool_load(*store, d0.w_gate, d0.w_up, d0.w_down, mv_list, mv_slot, mv_n, n_move, shape.H, shape.F)
            torch.cuda.synchronize()
            B.moe_profile_enable(True)
            for t in range(20):
                B.moe_pool_load(*store, d0.w_gate, d0.w_up, d0.w_down, mv_list, mv_slot, mv_n, n_move, shape.H, shape.F)
            torch.cuda.synchronize()
            B.moe_profile_enable(False)
            load_ms, load_n = B.moe_profile_read(B.KERNEL_POOL_LOAD)
            for w, sv in zip((d0.w_gate, d0.w_up, d0.w_down), saved):
                w[:n_move].copy_(sv)           # the pools go back to what the layer needs
            load_us = load_ms * 1e3 / load_n - ev_us
            moved = n_move * 6 * shape.H * shape.F
            overlap = None
            if not args.no_prefetch_overlap:
                # the paper's asynchronous prefetch (Sec. 3.4): the same copy, into a staging pool no layer reads,
                # on a second stream (default priority) while the verify steps run; one copy per verify step
                stage = [torch.empty_like(sv) for sv in saved]
                side = torch.cuda.Stream()
                n_ov = 120

                def chain(with_prefetch):
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    for i in range(n_ov):
                        step(i)
                        if with_prefetch:
                            B.moe_pool_load(*store, *stage, mv_list, mv_slot, mv_n, n_move, shape.H, shape.F, stream=side)
                    torch.cuda.synchronize()
                    us = (time.perf_counter() - t0) / n_ov * 1e6
                    healthy(buf.workspace, "verify steps beside the cache manager's copy")
                    return us

                chain(True)
                us_alone, us_with = chain(False), chain(True)
                # ... and with the store where the paper keeps it: pinned host memory the device reads directly
                host_store = [w.cpu().pin_memory() for w in store]
                dev_store, store = store, host_store
                B.moe_pool_load(*store, *stage, mv_list, mv_slot, mv_n, n_move, shape.H, shape.F)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for t in range(5):
                    B.moe_pool_load(*store, *stage, mv_list, mv_slot, mv_n, n_move, shape.H, shape.F)
                torch.cuda.synchronize()
                host_load_us = (time.perf_counter() - t0) / 5 * 1e6
                # the copy takes many verify steps: keep one in flight on the second stream all the time
                def chain_host():
                    torch.cuda.synchronize()
                    done = torch.cuda.Event()
                    n_loads = 0
                    t0 = time.perf_counter()
                    for i in range(4 * n_ov):
                        step(i)
                        if n_loads == 0 or done.query():
                            B.moe_pool_load(*store, *stage, mv_list, mv_slot, mv_n, n_move, shape.H, shape.F, stream=side)
                            done.record(side)
                            n_loads += 1
                    torch.cuda.current_stream().synchronize()
                    us = (time.perf_counter() - t0) / (4 * n_ov) * 1e6
                    torch.cuda.synchronize()
                    healthy(buf.workspace, "verify steps beside the cache manager's copy from pinned host memory")
                    return us, n_loads
                us_with_host, host_loads = chain_host()
                store = dev_store
                overlap = {"us_per_layer_alone": round(us_alone, 2),
                           "us_per_layer_with_one_load_per_step_on_a_second_stream": round(us_with, 2),
                           "bytes_loaded_per_step": moved,
                           "note": "the copy moves 2x its bytes through HBM; alone it takes load_kernel.avg_us",
                           "store_in_pinned_host_memory": {
                               "load_us_alone": round(host_load_us, 1),
                               "load_GBs": round(moved / host_load_us / 1e3, 1),
                               "us_per_layer_with_a_load_always_in_flight": round(us_with_host, 2),
                               "loads_started_during_%d_steps" % (4 * n_ov): host_loads}}
            est["cache_manager"] = {
                "plan_kernel": {"avg_us": round(plan_ms * 1e3 / plan_n - ev_us, 2), "layers": L_est, "bound": "latency"},
                "load_kernel": {"avg_us": round(load_us, 2), "experts": n_move, "bytes_moved": moved,
                                "bound": "hbm", "achieved_GBs_read_plus_write": round(2 * moved / load_us / 1e3, 1),
                                "frac_of_8TBs": round(2 * moved / load_us / 1e3 / HBM_PEAK_GBS, 4),
                                "store": "device memory"},
                "prefetch_overlap": overlap}
        if not args.no_cpu_baseline:
            import oracle
            z = np.zeros(shape.E, dtype=np.int32)
            th = np.full(shape.E, gamma // 2, dtype=np.int32)
            o_st = [(z.copy(), z.copy(), th.copy(), th.copy()) for _ in range(L_est)]
            tabs = d_tab.cpu().numpy()
            t_c0 = time.perf_counter()
            reps = 50
            for t in range(reps):
                for l in range(L_est):
                    o_st[l] = oracle.utility_step(fr[t % 8, l], *o_st[l], K_est, 1, 10)
                    oracle.prefetch_counts(o_st[l][1], tabs[l], K_est)
            est["cpu_oracle_us"] = round((time.perf_counter() - t_c0) * 1e6 / reps, 1)

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        li = layers[0]
        threads = oracle.max_threads()
        oracle.layer_from_inputs(li)  # warm-up
        n, t_cpu0 = 0, time.perf_counter()
        while True:
            oracle.layer_from_inputs(li)
            n += 1
            el = time.perf_counter() - t_cpu0
            if el >= args.cpu_seconds or n >= 5000:
                break
        cpu_s = el / n
        # ... and on a single thread (a few runs: one takes ~16 times as long)
        oracle.set_threads(1)
        n1, t1 = 0, time.perf_counter()
        while True:
            oracle.layer_from_inputs(li)
            n1 += 1
            el1 = time.perf_counter() - t1
            if el1 >= args.cpu_seconds / 3 or n1 >= 5000:
                break
        oracle.set_threads(threads)
        cpu = {"value": round(layer_bytes[0] / cpu_s / 1e9, 3), "unit": "GB/s", "cores": threads,
               "kind": "oracle", "us_per_layer": round(cpu_s * 1e6, 1),
               "sample": f"{n} runs of the whole layer 0 of this workload ({el:.1f}s), fp64 scalar C, "
                         f"OpenMP over output rows",
               "one_thread": {"value": round(layer_bytes[0] / (el1 / n1) / 1e9, 3), "us_per_layer": round(el1 / n1 * 1e6, 1),
                              "runs": n1}}

    out = {
        "metric": "verify-step MoE layer: expert-weight HBM GB/s (us per layer = 1000*ms_per_step), 1xMI355X",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "us_per_layer": round(ms_per_step * 1e3, 2),
        "whole_layer_frac": round(gbs / HBM_PEAK_GBS, 4),
        "timer": "host wall clock between two device synchronisations around the K steps, inputs resident in HBM",
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic", "launch": "hip graph replay" if args.graph else "eager",
        "config": {"workload": desc, "layers": len(layers), "launch_form": args.form,
                   "mean_weight_bytes_per_layer": int(np.mean(layer_bytes))},
        "roofline": roofline, "cpu_baseline": cpu, "north_star_rows": rows, "launch_forms": launch_forms,
        "estimator": est,
        # (the same object as estimator.cache_manager.prefetch_overlap: verify steps beside the cache manager's copy)
        "prefetch_overlap": (est or {}).get("cache_manager", {}).get("prefetch_overlap"),
    }
    if args.timeline:
        print_timeline(B, torch, np, step, len(layers))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
