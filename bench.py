#!/usr/bin/env python3
"""Benchmark of the HGF linear hot path on one MI355X.

A step is one pass of the whole path (activation quantiser, rank-r down-projection,
main kernel with fused epilogue, for every linear of the workload) through
hgf_stack_forward, on seeded synthetic inputs already resident in HBM.

Default workload: the 7B-shape FFN decode at M=1 (up, gate: 4096->11008; down:
11008->4096; r=128) over 32 distinct weight instances chained block to block, 1.46 GB of
parameters per step, so every step streams its weights from HBM (nothing fits in cache).
`value` is the achieved HBM GB/s over the algorithmic bytes of the step.  The same JSON
line also carries: tokens/s, the roofline record of the main decode kernel (its duration
measured with HIP events on the launch stream in a second pass), the CPU oracle timed on
a bounded sample, and secondary cases (the 8-layer d=512 stack at M=1, the 1.2B-shape
layer at M=1, the 3B-shape prefill layer at M=2048).
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
        self.stack = hb.Stack(self.layers, slots, M)
        self.bytes = sum(linear_bytes(K, N, r, M) for K, N, r in self.shapes)
        self.main_bytes = sum(main_kernel_bytes(K, N, r, M) for K, N, r in self.shapes)
        self.int8_ops = sum(2.0 * M * K * N for K, N, _ in self.shapes)
        self.param_bytes = sum(K * N / 4 + 2 * r * (K + N) + 2 * N + 4 for K, N, r in self.shapes)


def time_steps(fn, steps: int, warmup: int) -> float:
    """Seconds per step: `warmup` untimed calls, then exactly `steps` calls between two syncs."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


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
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-secondary", action="store_true", help="skip the secondary cases")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--target-wgs", type=int, default=0, help="decode workgroups per launch (0 = library default)")
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
    if args.target_wgs:
        hb.hgf_set_decode_target_workgroups(args.target_wgs)
    use_graph = not args.no_graph

    ws = hb.Workspace(2048, 11008, 11008, 128)

    # ---- primary: 7B-shape FFN decode, M = 1, distinct weights every block (HBM-cold)
    wl = Workload(4, 1, args.blocks, seed=4000, ws=ws)
    run = make_runner(wl, ws, use_graph)
    sec = time_steps(run, args.steps, args.warmup)
    gbs = wl.bytes / sec / 1e9
    (dms, dn), _ = kernel_profile(wl, ws, max(2, min(args.steps, 10)))    # a launch covers up+gate or down
    avg_kernel_s = dms / 1e3 / max(dn, 1)
    k_bytes = wl.main_bytes * max(2, min(args.steps, 10)) / max(dn, 1)   # algorithmic bytes per main-kernel launch
    achieved = k_bytes / avg_kernel_s / 1e9 if dn else 0.0

    out = {
        "metric": "HGF linear achieved HBM GB/s at M=1 (7B-shape FFN decode)",
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
            "workload": f"config 4 (7B-shape): up, gate 4096->11008 and down 11008->4096, r=128, M=1, "
                        f"{args.blocks} chained blocks of distinct weights via hgf_stack_forward",
            "linears_per_step": len(wl.layers),
            "algorithmic_bytes_per_step": int(wl.bytes),
            "launch": "hip-graph replay" if use_graph else "eager",
        },
        "roofline": {
            "kernel": "decode_kernel<1> (grouped main kernel: up+gate in one launch, down in the next)",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": None,
            "avg_launch_us": round(avg_kernel_s * 1e6, 3),
            "launches_timed": int(dn),
            "algorithmic_bytes_per_launch": int(k_bytes),
        },
    }

    if not args.no_cpu:
        cb = cpu_baseline(4, 1, 3, args.cpu_seconds)
        out["cpu_baseline"] = {
            "value": round(cb["bytes"] / cb["seconds_per_pass"] / 1e9, 3),
            "unit": "GB/s",
            "cores": cb["cores"],
            "kind": "oracle",
            "sample": f"one block (up, gate, down) of the workload at M=1, {cb['passes']} passes in "
                      f"{cb['passes'] * cb['seconds_per_pass']:.1f} s; a {args.blocks}-block step would take "
                      f"{cb['seconds_per_pass'] * args.blocks * 1e3:.0f} ms",
        }

    if not args.no_secondary:
        cases = {}
        del run, wl
        torch.cuda.empty_cache()
        # 8-layer d=512 stack at M=1: 14.7 MB of parameters, cache-resident ("hot"), launch bound
        w1 = Workload(1, 1, 8, seed=1000, ws=ws)
        s1 = time_steps(make_runner(w1, ws, use_graph), max(10, args.steps), args.warmup)
        cases["config1_stack_M1_hot"] = {"tokens_per_s": round(1.0 / s1, 1), "us_per_token": round(s1 * 1e6, 2),
                                         "linears": len(w1.layers),
                                         "GB_per_s_cache_resident": round(w1.bytes / s1 / 1e9, 1)}
        del w1
        # 1.2B-shape layer, M=1, 16 distinct blocks of 7 projections (cold)
        w2 = Workload(2, 1, 16, seed=2000, ws=ws)
        s2 = time_steps(make_runner(w2, ws, use_graph), max(10, args.steps // 2), args.warmup)
        cases["config2_layer_M1_cold"] = {"GB_per_s": round(w2.bytes / s2 / 1e9, 1),
                                          "frac_of_hbm_peak": round(w2.bytes / s2 / 1e9 / HBM_PEAK_GBS, 4),
                                          "us_per_layer": round(s2 / 16 * 1e6, 2)}
        del w2
        torch.cuda.empty_cache()
        # 3B-shape prefill layer, M=2048, the 7 projections of one block
        w3 = Workload(3, 2048, 1, seed=3000, ws=ws)
        s3 = time_steps(make_runner(w3, ws, False), 3, 1)
        (_, _), (pms, pn) = kernel_profile(w3, ws, 2)
        tops = w3.int8_ops / s3 / 1e12
        k_tops = w3.int8_ops / len(w3.layers) / (pms / 1e3 / max(pn, 1)) / 1e12 if pn else 0.0
        cases["config3_prefill_M2048"] = {"int8_TOPS": round(tops, 1), "frac_of_int8_peak": round(tops / INT8_PEAK_TOPS, 4),
                                          "ms_per_layer": round(s3 * 1e3, 3),
                                          "main_kernel_int8_TOPS": round(k_tops, 1)}
        out["cases"] = cases

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
