#!/usr/bin/env python3
"""Benchmark of the HGF linear hot path on one MI355X.

A step is one pass of the whole path (activation quantiser, rank-r down-projection,
main kernel with fused epilogue, for every linear of the workload) through
hgf_stack_forward, on seeded synthetic inputs already resident in HBM.

Default workload: the 7B-shape FFN decode at M=1 (up, gate: 4096->11008; down:
11008->4096; r=128) over 32 distinct weight instances chained block to block, 1.46 GB of
parameters per step, so every step streams its weights from HBM (nothing fits in cache).
`value` is the achieved HBM GB/s over the algorithmic bytes of the step.  The same JSON
line also carries: tokens/s, the roofline record of the decode kernel (one persistent
launch per run of layers, two per step; its duration measured with HIP events on the
launch stream; its HBM traffic from the committed counter summary under profiles/), the CPU oracle timed on a bounded sample, and secondary cases (the
8-layer d=512 stack at M=1, the 1.2B-shape layer at M=1, the 3B-shape prefill layer at
M=2048).

`--copy-probe MIB` instead runs a plain elementwise copy of that many MiB a few times:
the kernel of known size against which the HBM counters are scaled.
`--mfma-probe` instead prints what a loop of nothing but the prefill kernel's MFMA sustains
on constant, ternary-code x random and random operands (the chip's clock gives way under the
matrix cores' power): the practical ceiling beside the published int8 peak.
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

import numpy as np
import torch

from paper_2602_05269_amd import binding as hb
from paper_2602_05269_amd import build as hipbuild
from paper_2602_05269_amd import synth

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0     # MI355X dense int8 MFMA, published


def linear_bytes(K: int, N: int, r: int, M: int) -> float:
    """Algorithmic bytes of one HGF linear: packed T, A, B, alpha, s_w, x read once, y written once."""
    return K * N / 4 + 2 * r * (K + N) + 2 * N + 4 + 2 * M * K + 2 * M * N


def main_kernel_bytes(K: int, N: int, r: int, M: int) -> float:
    """The main kernel's share: everything but A (read by the down-projection kernel)."""
    return linear_bytes(K, N, r, M) - 2 * r * K


class Workload:
    """A layer list on the device built from a configuration's shapes and distributions."""

    def __init__(self, cfg: int, M: int, n_blocks: int, seed: int, ws: hb.Workspace, names=None):
        c = synth.CONFIGS[cfg]
        self.cfg, self.M, self.n_blocks = cfg, M, n_blocks
        wiring, _ = synth.stack_wiring(cfg, chained=True, n_layers=n_blocks)
        if names is not None:
            keep = {i for i, p in enumerate(c.projections) if p.name in names}
            wiring = [w for w in wiring if w[1] in keep]
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed)
        n_slots = 1 + max(w[3] for w in wiring)
        slots = [None] * n_slots
        x0 = synth.make_activations(cfg, 0, wiring[0][1], M)
        slots[0] = torch.from_numpy(x0).cuda()
        self.layers, self.shapes = [], []
        for (_layer, proj, src, dst) in wiring:
            p = c.projections[proj]
            W = torch.randn((p.d_out, p.d_in), generator=gen, device="cuda", dtype=torch.float32) * 0.02
            A = (torch.randn((c.rank, p.d_in), generator=gen, device="cuda") * c.lora_std).half()
            B = (torch.randn((p.d_out, c.rank), generator=gen, device="cuda") * c.lora_std).half()
            alpha = torch.randn(p.d_out, generator=gen, device="cuda").half()
            self.layers.append(hb.Layer.from_latent(W, A, B, alpha, ws, src_slot=src, dst_slot=dst))
            del W
            if slots[src] is None:      # a filtered-out producer: feed a fresh synthetic input
                slots[src] = torch.from_numpy(synth.make_activations(cfg, 0, proj, M)).cuda()
            slots[dst] = torch.zeros((M, p.d_out), dtype=torch.float16, device="cuda")
            self.shapes.append((p.d_in, p.d_out, c.rank))
        self.wiring, self.proj_of = wiring, [w[1] for w in wiring]
        self._finish(slots, M)

    def _finish(self, slots, M):
        self.M, self.slots = M, slots
        self.stack = hb.Stack(self.layers, slots, M)
        self.bytes = sum(linear_bytes(K, N, r, M) for K, N, r in self.shapes)
        self.main_bytes = sum(main_kernel_bytes(K, N, r, M) for K, N, r in self.shapes)
        self.int8_ops = sum(2.0 * M * K * N for K, N, _ in self.shapes)
        self.param_bytes = sum(K * N / 4 + 2 * r * (K + N) + 2 * N + 4 for K, N, r in self.shapes)

    def with_tokens(self, M: int) -> "Workload":
        """The same weights and wiring at another number of tokens (fresh input and slots)."""
        import copy
        other = copy.copy(self)
        c = synth.CONFIGS[self.cfg]
        slots = [None] * len(self.slots)
        slots[0] = torch.from_numpy(synth.make_activations(self.cfg, 0, self.wiring[0][1], M)).cuda()
        for (_layer, proj, src, dst) in self.wiring:
            if slots[src] is None:
                slots[src] = torch.from_numpy(synth.make_activations(self.cfg, 0, proj, M)).cuda()
            slots[dst] = torch.zeros((M, c.projections[proj].d_out), dtype=torch.float16, device="cuda")
        other._finish(slots, M)
        return other


def time_steps(fn, steps: int, warmup: int, events: bool = False):
    """Seconds per step: `warmup` untimed calls, then exactly `steps` calls between two syncs.
    With `events`, also the seconds per step between two HIP events recorded on the launch
    stream (torch's current stream, which the binding launches on) around the same calls."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    return (wall, e0.elapsed_time(e1) / 1e3 / steps) if events else wall


def make_runner(wl: Workload, ws: hb.Workspace, use_graph: bool):
    """Returns fn() that enqueues one step on torch's current stream."""
    if not use_graph:
        return lambda: hb.hgf_stack_forward(wl.stack, ws)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        hb.hgf_stack_forward(wl.stack, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        hb.hgf_stack_forward(wl.stack, ws)
    torch.cuda.synchronize()
    wl._graph = graph
    return graph.replay


def kernel_profile(wl: Workload, ws: hb.Workspace, steps: int):
    """Average main-kernel launch duration (ms) from HIP events on the launch stream."""
    hb.hgf_stack_forward(wl.stack, ws)
    torch.cuda.synchronize()
    hb.hgf_profile_enable(True)
    try:
        for _ in range(steps):
            hb.hgf_stack_forward(wl.stack, ws)
        torch.cuda.synchronize()
        (dms, dn), (pms, pn) = hb.hgf_profile_collect()
    finally:
        hb.hgf_profile_enable(False)
    return (dms, dn), (pms, pn)


TRAFFIC_FILE = os.path.join(ROOT, "profiles", "decode_m1_config4_hbm_traffic.txt")


def recorded_traffic():
    """HBM bytes per decode launch from the committed counter summary (None if absent)."""
    try:
        for line in open(TRAFFIC_FILE):
            if line.startswith("traffic_bytes_per_launch"):
                return int(float(line.split("=")[1].split()[0]))
    except OSError:
        pass
    return None


def timeline(wl: Workload, ws: hb.Workspace, ph0: int) -> int:
    """Medians over the workgroups of the in-kernel time stamps of phases ph0 .. ph0+3 of the first
    whole-stack launch of a step, in microseconds after the moment the last workgroup stored the
    last output of the phase before (the earliest moment the phase's input is complete)."""
    for _ in range(3):
        hb.hgf_stack_forward(wl.stack, ws)
    torch.cuda.synchronize()
    plain = time_steps(lambda: hb.hgf_stack_forward(wl.stack, ws), 10, 2)
    buf = torch.zeros((256, hb.TRACE_ROLES, hb.TRACE_PHASES, hb.TRACE_IDS), dtype=torch.int64, device="cuda")
    hb.hgf_set_stack_trace(buf, ph0)
    try:
        traced = time_steps(lambda: hb.hgf_stack_forward(wl.stack, ws), 10, 2)
        buf.zero_()
        torch.cuda.synchronize()
        hb.hgf_stack_forward(wl.stack, ws)
        torch.cuda.synchronize()
    finally:
        hb.hgf_set_stack_trace(None)
    t = buf.cpu().numpy().astype(np.float64) / 100.0          # 100 MHz clock -> microseconds
    t[t == 0] = np.nan
    # NOTE: a step is two launches; the second overwrites the first's stamps, both walk the same shapes
    print(f"ms per step: {plain * 1e3:.4f} without stamps, {traced * 1e3:.4f} with")
    names = {"contract": ["enter", "tokens complete", "absmax agreed", "quantised", "first unit contracted", "last unit contracted"],
             "slice": ["enter", "own slices stored", "SiLU(A x) in LDS", "own slice multiplied"],
             "unit": ["enter", "SiLU(A x) seen", "first unit complete", "last unit complete", "last unit stored",
                      "first unit's B h done"]}
    raw = buf.cpu().numpy().astype(np.float64)
    dclk = raw[:, 10, 3, 2] - raw[:, 10, 0, 2]
    dwall = (raw[:, 10, 3, 0] - raw[:, 10, 0, 0]) / 100.0
    print(f"shader clock over the traced phases: {float(np.nanmedian(dclk / dwall)):.0f} MHz")
    for k in range(1, hb.TRACE_PHASES):
        ph = ph0 + k
        prev_done = np.nanmax(t[:, 9, k - 1, 4])
        this_done = np.nanmax(t[:, 9, k, 4])
        busy = ~np.isnan(t[:, 9, k, 2])
        print(f"phase {ph}: {int(busy.sum())} workgroups own units; {this_done - prev_done:.2f} us from the last store "
              f"of phase {ph - 1} to the last store of phase {ph}")
        rel = t[busy] - prev_done
        med = lambda a: float(np.nanmedian(a))
        c = rel[:, 0:8, k, :]
        print("  contracting wavefronts (per workgroup: first / last of the eight; then the median over workgroups)")
        for i, nm in enumerate(names["contract"]):
            print(f"    {nm:24s} first {med(np.nanmin(c[:, :, i], axis=1)):6.2f}   last {med(np.nanmax(c[:, :, i], axis=1)):6.2f}")
        waited = raw[busy][:, 0:8, k, 6] / 100.0
        print(f"    waits for weight tiles   {float(np.median(np.sum(raw[busy][:, 0:8, k, 7], axis=1))):6.0f} per workgroup, "
              f"{float(np.median(np.max(waited, axis=1))):5.2f} us in the wavefront that waited longest (median; "
              f"mean over wavefronts {float(np.median(np.mean(waited, axis=1))):5.2f} us)")
        for i, nm in enumerate(names["slice"]):
            print(f"  slice wavefront  {nm:22s} {med(rel[:, 8, k, i]):6.2f}")
        allrel = t - prev_done
        has = ~np.isnan(allrel[:, 8, k, 3])
        if has.any():
            print(f"  slice wavefronts with a slice ({int(has.sum())}): last slice multiplied {med(allrel[has, 8, k, 3]):6.2f} "
                  f"(latest {float(np.nanmax(allrel[has, 8, k, 3])):6.2f}), stored {med(allrel[has, 8, k, 1]):6.2f} "
                  f"(latest {float(np.nanmax(allrel[has, 8, k, 1])):6.2f})")
        for i, nm in enumerate(names["unit"]):
            print(f"  unit wavefront   {nm:22s} {med(rel[:, 9, k, i]):6.2f}   (latest workgroup {float(np.nanmax(rel[:, 9, k, i])):6.2f})")
        print(f"  loader 0         first tile requested  {med(rel[:, 10, k, 0]):6.2f}   last {med(rel[:, 10, k, 1]):6.2f}")
    return 0


def mfma_probe() -> int:
    """The yardstick beside the published int8 peak: what the matrix cores sustain on this
    layer's kind of operands once the chip has settled its clock under their power."""
    torch.cuda.set_device(0)
    out = {"probe": "v_mfma_i32_32x32x32_i8 only, 8 accumulators, 2 workgroups x 4 wavefronts per compute unit",
           "published_peak_TOPS": INT8_PEAK_TOPS}
    for kind, name in ((0, "constant"), (1, "codes_0_2_x_random_int8"), (2, "random_int8")):
        tops, ghz = hb.hgf_probe_mfma_rate(kind, 800)
        out[name] = {"TOPS": round(tops, 1), "clock_GHz": round(ghz, 3)}
    print(json.dumps(out))
    return 0


def copy_probe(mib: int) -> int:
    """A plain copy of `mib` MiB (read once, written once) by an elementwise kernel, five times."""
    n = mib * (1 << 20) // 4
    src = torch.arange(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(5):
        torch.mul(src, 1.0, out=dst)
    torch.cuda.synchronize()
    print(json.dumps({"copy_probe_bytes_read": n * 4, "copy_probe_bytes_written": n * 4, "launches": 5}))
    return 0


def cpu_baseline(cfg: int, M: int, n_linears: int, budget_s: float):
    """The CPU oracle, as it stands, on the first `n_linears` projections of the workload
    (same shapes and distributions, host-generated), repeated until ~budget_s has elapsed."""
    from oracle import hgf_oracle as orc
    c = synth.CONFIGS[cfg]
    cases = []
    for i in range(n_linears):
        proj = i % len(c.projections)
        w = synth.make_weights(cfg, i // len(c.projections), proj)
        T, s_w = orc.ternarize(w["W"])
        x = synth.make_activations(cfg, 0, proj, M)
        cases.append((x, T, s_w, w["A"], w["B"], w["alpha"]))
        del w
    nbytes = sum(linear_bytes(T.shape[1], T.shape[0], A.shape[0], M) for (_, T, _, A, _, _) in cases)
    ops = sum(2.0 * M * T.shape[1] * T.shape[0] for (_, T, _, _, _, _) in cases)
    orc.linear_forward(*cases[0])                      # warm the library
    t0 = time.perf_counter()
    passes = 0
    while True:
        for cse in cases:
            orc.linear_forward(*cse)
        passes += 1
        el = time.perf_counter() - t0
        if el >= budget_s or passes >= 1000:
            break
    per_pass = el / passes
    return {"seconds_per_pass": per_pass, "bytes": nbytes, "ops": ops, "passes": passes,
            "cores": orc.num_threads()}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--blocks", type=int, default=32, help="distinct weight instances (FFN blocks) per step")
    ap.add_argument("--tokens", type=int, default=1,
                    help="tokens M of the primary workload (default 1, the headline metric; other values are "
                         "for profiling the few-token paths)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-secondary", action="store_true", help="skip the secondary cases")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--mfma-probe", action="store_true",
                    help="print the int8 rate a loop of nothing but the prefill kernel's MFMA sustains, "
                         "for constant, ternary-code x random and random operands, and exit")
    ap.add_argument("--timeline", type=int, default=-1, metavar="PHASE",
                    help="print the time line of four phases of the whole-stack launch from this phase on "
                         "(time stamps taken inside the kernel) and exit")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MIB",
                    help="run only a plain copy kernel of this many MiB (counter calibration)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the HGF linear path has no multi-GPU part); "
              "run with --gpus 1", file=sys.stderr)
        return 2
    if not os.path.exists(hb.LIB_PATH):
        hipbuild.build(force=True)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.copy_probe:
        return copy_probe(args.copy_probe)
    if args.mfma_probe:
        return mfma_probe()
    use_graph = not args.no_graph

    ws = hb.Workspace(2048, 11008, 11008, 128)

    # ---- primary: 7B-shape FFN decode, M = 1, distinct weights every block (HBM-cold)
    wl = Workload(4, args.tokens, args.blocks, seed=4000, ws=ws)
    if args.timeline >= 0:
        return timeline(wl, ws, args.timeline)
    run = make_runner(wl, ws, use_graph)
    sec, ev_sec = time_steps(run, args.steps, args.warmup, events=True)
    gbs = wl.bytes / sec / 1e9
    # The decode kernel is the only kernel of a step: one persistent launch per run of layers
    # (as many as one launch's description holds: 16 FFN blocks, so two launches per step).
    # Its average launch duration over the timed region is the region's length between two
    # HIP events on the launch stream divided by the launches in it (gaps between launches
    # count against the kernel).  A second, eager pass brackets every launch with its own
    # event pair and is reported aside.
    psteps = max(2, min(args.steps, 10))
    (dms, dn), _ = kernel_profile(wl, ws, psteps)
    launches_per_step = max(dn // psteps, 1)
    avg_kernel_s = ev_sec / launches_per_step
    k_bytes = wl.bytes / launches_per_step                               # algorithmic bytes per launch
    achieved = k_bytes / avg_kernel_s / 1e9

    out = {
        "metric": f"HGF linear achieved HBM GB/s at M={args.tokens} (7B-shape FFN decode)",
        "value": round(gbs, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 x ternary -> int32, fp16 correction (fp32 accumulate)",
        "data": "synthetic",
        "tokens_per_s": round(1.0 / sec, 1),
        "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
        "config": {
            "workload": f"config 4 (7B-shape): up, gate 4096->11008 and down 11008->4096, r=128, M={args.tokens}, "
                        f"{args.blocks} chained blocks of distinct weights via hgf_stack_forward (a pure chain of "
                        f"linears: no norms or residuals, so the values drift block by block -- see chain_end; "
                        f"the kernels' time does not depend on the values)",
            "linears_per_step": len(wl.layers),
            "algorithmic_bytes_per_step": int(wl.bytes),
            "launch": "hip-graph replay" if use_graph else "eager",
        },
        "roofline": {
            "kernel": "stack_kernel (one persistent launch per run of 16 FFN blocks = 32 groups of layers)",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": recorded_traffic(),
            "avg_launch_us": round(avg_kernel_s * 1e6, 3),
            "launches_timed": int(launches_per_step * args.steps),
            "algorithmic_bytes_per_launch": int(k_bytes),
            "per_launch_event_pairs_us": round(dms * 1e3 / max(dn, 1), 3),
        },
    }

    if not args.no_cpu:
        cb = cpu_baseline(4, args.tokens, 3, args.cpu_seconds)
        out["cpu_baseline"] = {
            "value": round(cb["bytes"] / cb["seconds_per_pass"] / 1e9, 3),
            "unit": "GB/s",
            "cores": cb["cores"],
            "kind": "oracle",
            "sample": f"one block (up, gate, down) of the workload at M={args.tokens}, {cb['passes']} passes in "
                      f"{cb['passes'] * cb['seconds_per_pass']:.1f} s; a {args.blocks}-block step would take "
                      f"{cb['seconds_per_pass'] * args.blocks * 1e3:.0f} ms",
        }

    if not args.no_secondary and args.tokens == 1:
        cases = {}
        hbm = lambda nbytes, s_: {"us": round(s_ * 1e6, 2), "algorithmic_bytes": int(nbytes),
                                  "GB_per_s": round(nbytes / s_ / 1e9, 1),
                                  "frac_of_hbm_peak": round(nbytes / s_ / 1e9 / HBM_PEAK_GBS, 4)}
        few = max(5, args.steps // 5)
        # what the chain's values have become at its end (no norms or residuals between the linears)
        last = wl.slots[wl.wiring[-1][3]].float()
        out["config"]["chain_end"] = {"absmax": float(last.abs().nan_to_num(nan=0.0, posinf=65504.0).max()),
                                      "non_finite": int((~torch.isfinite(last)).sum())}
        # ---- config 4 at more tokens: the same 32 blocks of weights (cold), per FFN block
        cases["config4_block_M1_cold"] = hbm(wl.bytes / args.blocks, sec / args.blocks)
        for M in (2, 4, 8, 32, 64):
            wm = wl.with_tokens(M)
            sm = time_steps(make_runner(wm, ws, use_graph), few, 2)
            c = hbm(wm.bytes / args.blocks, sm / args.blocks)
            c["path"] = "whole-stack launches (stack_kernel)" if M <= 4 else \
                        "two-launch decode (prologue_kernel, decode_kernel)" if M <= 40 else \
                        "up + gate: prefill path (prepare_kernel, prefill_kernel); down: two-launch decode"
            cases[f"config4_block_M{M}_cold"] = c
            del wm

        # ---- the fused SwiGLU pair (gate and up of one input -> z) on the same weights, against
        #      the two layers as one group with two outputs
        def pair_time(M, fused):
            x = torch.from_numpy(synth.make_activations(4, 0, 0, M)).cuda()
            ups = [l for l, p_ in zip(wl.layers, wl.proj_of) if p_ == 0]
            gates = [l for l, p_ in zip(wl.layers, wl.proj_of) if p_ == 1]
            z = torch.zeros((M, ups[0].d_out), dtype=torch.float16, device="cuda")
            z2 = torch.zeros_like(z)
            stacks = []
            for u, g in zip(ups, gates):
                a = hb.Layer(u.packed, u.s_w, u.d_out, u.d_in, u.A, u.B, u.alpha, src_slot=0, dst_slot=1)
                b = hb.Layer(g.packed, g.s_w, g.d_out, g.d_in, g.A, g.B, g.alpha, src_slot=0, dst_slot=2)
                stacks.append(hb.Stack([a, b], [x, z, z2], M))

            def step():
                for u, g, st in zip(ups, gates, stacks):
                    if fused:
                        hb.hgf_swiglu_forward(x, g, u, ws, z=z)
                    else:
                        hb.hgf_stack_forward(st, ws)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                step()
            torch.cuda.synchronize()
            t = time_steps(graph.replay, few, 2) / len(ups)
            K, N, r = ups[0].d_in, ups[0].d_out, ups[0].rank
            nbytes = 2 * linear_bytes(K, N, r, M) - 2 * M * K - (2 * M * N if fused else 0)
            return hbm(nbytes, t)
        for M in (1, 8, 64):
            cases[f"config4_swiglu_pair_M{M}_cold"] = pair_time(M, True)
            cases[f"config4_up_gate_group_M{M}_cold"] = pair_time(M, False)
        del run, wl
        torch.cuda.empty_cache()

        # ---- base-3 packing (1.6 bits per weight) against the 2-bit layout: 16 distinct `up`
        #      layers (4096 -> 11008, r=128) at M=1, one call per layer.  "same_path": the 2-bit
        #      layer through the launch-per-step path as well (prologue, main kernel; the base-3 path has
        #      the slice reduction as a third launch).
        def b3_cases():
            gen = torch.Generator(device="cuda")
            gen.manual_seed(4500)
            K, N, r, nl = 4096, 11008, 128, 16
            l2, l3 = [], []
            for _ in range(nl):
                W = torch.randn((N, K), generator=gen, device="cuda", dtype=torch.float32) * 0.02
                A = (torch.randn((r, K), generator=gen, device="cuda") * 0.02).half()
                B = (torch.randn((N, r), generator=gen, device="cuda") * 0.02).half()
                alpha = torch.randn(N, generator=gen, device="cuda").half()
                l2.append(hb.Layer.from_latent(W, A, B, alpha, ws))
                p3, s3 = hb.hgf_quantize_pack_weights_b3(W, ws)
                l3.append(hb.Layer(p3, s3, N, K, A, B, alpha))
                del W
            x = torch.from_numpy(synth.make_activations(4, 0, 0, 1)).cuda()
            y = torch.zeros((1, N), dtype=torch.float16, device="cuda")

            def timed(fn):
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    fn()
                torch.cuda.current_stream().wait_stream(side)
                torch.cuda.synchronize()
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    fn()
                torch.cuda.synchronize()
                return time_steps(graph.replay, few, 2) / nl
            res = {}
            b2 = linear_bytes(K, N, r, 1)
            b3 = b2 - K * N / 4 + hb.hgf_packed_weight_bytes_b3(N, K)
            res["config4_up_M1_2bit_cold"] = hbm(b2, timed(lambda: [hb.hgf_linear_forward(x, l, ws, y=y) for l in l2]))
            hb.hgf_set_single_launch(0)
            try:
                res["config4_up_M1_2bit_same_path_cold"] = hbm(b2, timed(lambda: [hb.hgf_linear_forward(x, l, ws, y=y) for l in l2]))
            finally:
                hb.hgf_set_single_launch(2)
            res["config4_up_M1_base3_cold"] = hbm(b3, timed(lambda: [hb.hgf_linear_forward_b3(x, l, ws, y=y) for l in l3]))
            return res
        cases.update(b3_cases())
        torch.cuda.empty_cache()

        # ---- differential-attention decode step: the K and V caches are streamed once
        def attn_case(B, L, H, d_h):
            gen = torch.Generator(device="cuda")
            gen.manual_seed(4700)
            q = torch.randn((B, 2 * H, d_h), generator=gen, device="cuda").half()
            k = torch.randn((B, L, 2 * H, d_h), generator=gen, device="cuda").half()
            v = torch.randn((B, L, H, d_h), generator=gen, device="cuda").half()
            lens = torch.full((B,), L, dtype=torch.int32, device="cuda")
            o = torch.empty((B, H, d_h), dtype=torch.float16, device="cuda")
            wsp = torch.empty(hb.lib().hgf_diff_attention_workspace_bytes(B, L, H, d_h), dtype=torch.uint8, device="cuda")
            t = time_steps(lambda: hb.hgf_diff_attention_decode(q, k, v, lens, 0.8, out=o, workspace=wsp), 20, 3)
            return hbm(B * L * 3 * H * d_h * 2 + B * 3 * H * d_h * 2 + B * H * d_h * 2, t)
        cases["diff_attention_decode_d4096_h32_B8_L4096"] = attn_case(8, 4096, 32, 64)
        cases["diff_attention_decode_d512_h8_B64_L512"] = attn_case(64, 512, 8, 32)
        torch.cuda.empty_cache()
        # ---- config 0: the single 256x256 linear at 8 tokens (cache-resident, launch bound)
        w0 = Workload(0, 8, 1, seed=0, ws=ws)
        s0 = time_steps(make_runner(w0, ws, use_graph), max(20, args.steps), args.warmup)
        cases["config0_single_M8_hot"] = hbm(w0.bytes, s0)
        cases["config0_single_M8_hot"]["note"] = "0.03 MB of parameters: the latency of two launches, not bandwidth"
        del w0
        # 8-layer d=512 stack at M=1: 14.7 MB of parameters, cache-resident ("hot"), launch bound
        w1 = Workload(1, 1, 8, seed=1000, ws=ws)
        s1 = time_steps(make_runner(w1, ws, use_graph), max(10, args.steps), args.warmup)
        cases["config1_stack_M1_hot"] = {"tokens_per_s": round(1.0 / s1, 1), "us_per_token": round(s1 * 1e6, 2),
                                         "linears": len(w1.layers),
                                         "GB_per_s_cache_resident": round(w1.bytes / s1 / 1e9, 1)}
        del w1
        # 1.2B-shape layer, 16 distinct blocks of 7 projections (cold), per block
        w2 = Workload(2, 1, 16, seed=2000, ws=ws)
        for M in (1, 4, 16):
            wm = w2 if M == 1 else w2.with_tokens(M)
            s2 = time_steps(make_runner(wm, ws, use_graph), max(10, args.steps // 2), args.warmup)
            cases[f"config2_layer_M{M}_cold"] = hbm(wm.bytes / 16, s2 / 16)
        del w2, wm
        torch.cuda.empty_cache()
        # 3B-shape prefill layer, M=2048, the 7 projections of one block
        w3 = Workload(3, 2048, 1, seed=3000, ws=ws)
        s3 = time_steps(make_runner(w3, ws, False), 20, 3)
        (_, _), (pms, pn) = kernel_profile(w3, ws, 2)      # two passes; the events bracket grouped launches
        tops = w3.int8_ops / s3 / 1e12
        k_tops = 2 * w3.int8_ops / (pms / 1e3) / 1e12 if pn else 0.0
        cases["config3_prefill_M2048"] = {"int8_TOPS": round(tops, 1), "frac_of_int8_peak": round(tops / INT8_PEAK_TOPS, 4),
                                          "ms_per_layer": round(s3 * 1e3, 3),
                                          "main_kernel_int8_TOPS": round(k_tops, 1)}
        # the same block's gate and up projections as the fused SwiGLU pair (one output)
        names = [p_.name for p_ in synth.CONFIGS[3].projections]
        gi, ui = names.index("gate"), names.index("up")
        xg = w3.slots[w3.wiring[ui][2]]
        zz = torch.zeros((2048, w3.layers[ui].d_out), dtype=torch.float16, device="cuda")
        sp = time_steps(lambda: hb.hgf_swiglu_forward(xg, w3.layers[gi], w3.layers[ui], ws, z=zz), 20, 3)
        ops = 2 * 2.0 * 2048 * w3.layers[ui].d_in * w3.layers[ui].d_out
        cases["config3_swiglu_pair_M2048"] = {"int8_TOPS": round(ops / sp / 1e12, 1),
                                              "frac_of_int8_peak": round(ops / sp / 1e12 / INT8_PEAK_TOPS, 4),
                                              "us": round(sp * 1e6, 1)}
        out["cases"] = cases

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
