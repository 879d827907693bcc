#!/usr/bin/env python3
"""Throughput of one Union-of-Experts layer forward (uoe_layer_forward) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload lm|longrange|vit|large|tiny]

A step is one pass of the whole hot path (route -> SMHA -> route -> UoME) over one batch of seeded
synthetic input that is already resident in HBM.  Prints ONE JSON line with the whole-job
tokens/s, a roofline entry for the dominant kernel (timed live with events on the launch stream)
and the CPU oracle timed on this machine's host cores as a reported baseline.
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

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3    # MI355X fp32 vector/matrix
PEAK_HBM_GBS = 8000.0


def layer_flops(c) -> dict:
    """Algorithmic FLOPs of one layer call: active units only, no padding."""
    routers = 2 * c.b * c.l * c.d * (2 * c.n_a + c.n_m) + 2 * c.b * c.n_a * c.l * c.m   # both SMHA routers counted
    qkv = c.b * c.k_a * 6 * c.l_a * c.d * c.d_h
    attn = c.b * c.k_a * 4 * c.l_a * c.l_a * c.d_h
    outp = c.b * c.k_a * 2 * c.l_a * c.d_h * c.d
    uome = c.b * c.k_m * 4 * (c.c_m * (c.l // c.m_m)) * c.d * c.d_e   # rows an MLP expert sees: all of l unless data-selected
    return dict(routers=routers, qkv=qkv, attention=attn, out_proj=outp, uome=uome,
                total=routers + qkv + attn + outp + uome)


def describe(c) -> str:
    ds = f" m{c.m_m} c{c.c_m}" if c.m_m > 1 else ""
    return (f"{c.name}: b{c.b} l{c.l} d{c.d}; SMHA n{c.n_a} d_h{c.d_h} m{c.m} c{c.c} k{c.k_a}; "
            f"UoME n{c.n_m} d_e{c.d_e} k{c.k_m}{ds}; {c.dtype}")


def run_stage(args, cfg, dev, B, torch, make_lane) -> int:
    """Loop one stage (its inputs produced once by the stages before it) and print its mean time."""
    dev.layer_forward()      # fills routing results and u
    dev.smha_forward()
    dev.route_m()
    hidden = torch.empty((cfg.b, cfg.l, cfg.k_m * cfg.d_e), dtype=dev.tdtype, device=dev.device)
    h = torch.empty((cfg.b, cfg.k_a, cfg.l_a, cfg.d), dtype=dev.tdtype, device=dev.device)
    if cfg.m_m == 1:
        B.uome_up(dev.uome, dev.u, dev.a_in, dev.m_expert_idx, dev.m_expert_gate, hidden)
    calls = {
        "route_a": dev.route_a, "smha": dev.smha_forward, "route_m": dev.route_m, "uome": dev.uome_forward,
        "uome_up": lambda: B.uome_up(dev.uome, dev.u, dev.a_in, dev.m_expert_idx, dev.m_expert_gate, hidden),
        "uome_down": lambda: B.uome_down(dev.uome, hidden, dev.a_out, dev.u, dev.m_expert_idx, dev.out),
        "gather": lambda: B.gather(dev.smha, dev.x, dev.a_expert_idx, dev.a_patch_idx, h),
    }
    if args.stage == "uome_bwd":   # backward of the expert-selection UoME block on a synthetic upstream gradient
        from paper_2503_02495_amd import synth
        from paper_2503_02495_amd.harness import to_device
        d_out = to_device(synth.make_upstream_grad(cfg), cfg.dtype, dev.device)
        calls["uome_bwd"] = lambda: dev.uome_backward(d_out)
    if args.stage == "smha_bwd":   # backward of the SMHA block on a synthetic upstream gradient
        from paper_2503_02495_amd import synth
        from paper_2503_02495_amd.harness import to_device
        d_out_a = to_device(synth.make_upstream_grad(cfg), cfg.dtype, dev.device)
        calls["smha_bwd"] = lambda: dev.smha_backward(d_out_a)
    if args.stage in ("layer_bwd", "layer_fwd_bwd", "route_bwd"):
        from paper_2503_02495_amd import synth
        from paper_2503_02495_amd.harness import to_device
        d_out_l = to_device(synth.make_upstream_grad(cfg), cfg.dtype, dev.device)
        calls["layer_bwd"] = lambda: dev.layer_backward(d_out_l, u=dev.u)      # u kept from the forward pass

        def fwd_bwd():
            dev.layer_forward()
            dev.layer_backward(d_out_l)                                         # u recomputed (the layer call keeps it private)
        calls["layer_fwd_bwd"] = fwd_bwd
        if args.stage == "route_bwd":
            d_ge, d_gp = (to_device(t, synth.F32, dev.device) for t in synth.make_gate_grads(cfg, cfg.n_a, cfg.m))
            d_x = torch.empty_like(dev.x).copy_(d_out_l)
            grads = [torch.empty_like(t) for t in (dev.a_w_expert, dev.a_w_b, dev.a_w_a)]
            ws = torch.empty(B.route_backward_workspace_bytes(dev.smha), dtype=torch.uint8, device=dev.device)
            calls["route_bwd"] = lambda: B.route_backward(dev.smha, dev.x, dev.a_w_expert, dev.a_w_b, dev.a_w_a,
                                                          dev.a_expert_gate, dev.a_patch_gate, d_ge, d_gp, d_x, *grads, ws)
    if args.stage == "copy":   # a plain copy of known size (1 GiB read + 1 GiB written): counter calibration
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev.device).normal_()
        dst = torch.empty_like(src)
        calls["copy"] = lambda: dst.copy_(src)
    if args.stage == "lib_gemm":   # context only: the vendor library's plain batched GEMM (no expert lookup, no SiLU,
        # no gate, no residual) on the shapes of the two UoME GEMMs; nothing in the path calls it
        ncol = cfg.k_m * cfg.d_e
        ga = torch.empty((cfg.b, cfg.l, cfg.d), dtype=dev.tdtype, device=dev.device).normal_()
        gw1 = torch.empty((cfg.b, cfg.d, ncol), dtype=dev.tdtype, device=dev.device).normal_()
        gh = torch.empty((cfg.b, cfg.l, ncol), dtype=dev.tdtype, device=dev.device)
        gw2 = torch.empty((cfg.b, ncol, cfg.d), dtype=dev.tdtype, device=dev.device).normal_()
        go = torch.empty((cfg.b, cfg.l, cfg.d), dtype=dev.tdtype, device=dev.device)
        res = {}
        for nm, f in (("up_shape", lambda: torch.bmm(ga, gw1, out=gh)), ("down_shape", lambda: torch.bmm(gh, gw2, out=go))):
            for _ in range(args.warmup):
                f()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(args.steps):
                f()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / args.steps
            res[nm] = {"us_per_call": round(us, 3), "tflops": round(2.0 * cfg.b * cfg.l * cfg.d * ncol / us * 1e-6, 1)}
        print(json.dumps({"stage": "lib_gemm", "workload": cfg.name, "steps": args.steps, **res}))
        return 0
    if args.stage == "layer_fwd_bwd" and args.stage_streams > 1:
        # a training step per batch, several independent batches in flight (one lane per stream, lane 0 on the
        # program's own stream), as the forward benchmark does by default
        n_lanes = args.stage_streams
        lanes = [dev] + [make_lane() for _ in range(n_lanes - 1)]
        raw = [int(torch.cuda.current_stream().cuda_stream)] + [int(torch.cuda.Stream().cuda_stream) for _ in lanes[1:]]
        for lane in lanes:
            lane.layer_forward()
            lane.layer_backward(d_out_l)           # allocates the lane's gradient buffers
        torch.cuda.synchronize()

        def run(count):
            for i in range(count):
                lane, st = lanes[i % n_lanes], raw[i % n_lanes]
                lane.layer_forward(stream=st)
                lane.layer_backward(d_out_l, stream=st)
        run(max(args.warmup, n_lanes))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(args.steps)
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) * 1e6 / args.steps
        print(json.dumps({"stage": args.stage, "workload": cfg.name, "steps": args.steps, "streams": n_lanes,
                          "us_per_call": round(us, 3)}))
        return 0
    fn = calls[args.stage]
    for _ in range(args.warmup):
        fn()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(args.steps):
        fn()
    ev1.record()
    torch.cuda.synchronize()
    print(json.dumps({"stage": args.stage, "workload": cfg.name, "steps": args.steps,
                      "us_per_call": round(ev0.elapsed_time(ev1) * 1e3 / args.steps, 3)}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="lm")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--causal", action="store_true", help="SMHA with the shared causal mask (Sec. III-C.3)")
    ap.add_argument("--rope-dim", type=int, default=0, help="SMHA with partial RoPE on the last N dims (Eq. 32)")
    ap.add_argument("--uome-data-selection", default=None, metavar="M,C",
                    help="UoME with patch-wise data selection (Eq. 37): M patches, C kept per expert")
    ap.add_argument("--smha-mode", default="both", choices=["both", "expert", "data"],
                    help="selection modes of the SMHA block: both (default), expert selection only (c = m, no data "
                         "router) or data selection only (k = n, no expert router)")
    ap.add_argument("--dynamic-capacity", type=int, default=0, metavar="K",
                    help="two-stage routing (Eq. 15-16): every step first computes the SMHA capacity with K experts per "
                         "patch (uoe_route_capacity), reads it back and runs the layer with c = its maximum over the batch")
    ap.add_argument("--streams", type=int, default=4, metavar="S",
                    help="independent steps in flight: step i runs on HIP stream i %% S with its own inputs, workspace and "
                         "output (the steps of a throughput job do not depend on each other; one layer call is a chain of "
                         "nine dependent launches that leaves the GPU idle between them; the default is one lane per "
                         "hardware queue of the process: the stream the rest of the program uses and three more).  "
                         "1 = one call after the other; that figure is reported beside the headline either way")
    ap.add_argument("--stage-streams", type=int, default=1, metavar="S",
                    help="with --stage layer_fwd_bwd: S independent training steps in flight, one lane per stream")
    ap.add_argument("--graph", action="store_true",
                    help="replay one captured HIP graph per step instead of launching call by call")
    ap.add_argument("--stage", default=None,
                    choices=["route_a", "smha", "route_m", "uome", "uome_up", "uome_down", "gather", "copy",
                             "uome_bwd", "smha_bwd", "route_bwd", "layer_bwd", "layer_fwd_bwd", "lib_gemm"],
                    help="profiling aid: loop one C-ABI call of the path instead of the whole layer "
                         "and print its time (no JSON contract line)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2503_02495_amd import binding as B
    from paper_2503_02495_amd import synth
    from paper_2503_02495_amd.harness import DeviceLayer

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    B.lib()  # fail loudly if the HIP library is not built
    cfg = synth.CONFIGS[args.workload]
    uome_ds = args.uome_data_selection is not None
    if uome_ds:
        import dataclasses
        m_m, c_m = (int(v) for v in args.uome_data_selection.split(","))
        cfg = dataclasses.replace(cfg, m_m=m_m, c_m=c_m)
    if args.smha_mode != "both":
        import dataclasses
        cfg = dataclasses.replace(cfg, c=cfg.m) if args.smha_mode == "expert" else dataclasses.replace(cfg, k_a=cfg.n_a)
    inp = synth.make_inputs(cfg)
    inp.noise_m_patch = None   # the layer call takes no noise on the UoME patch logits
    if args.smha_mode == "expert":
        inp.a_w_b = inp.a_w_a = inp.noise_a_patch = None
    elif args.smha_mode == "data":
        inp.a_w_expert = inp.noise_a_expert = None
    fa = B.FLAG_RESIDUAL | (B.FLAG_CAUSAL if args.causal else 0)
    fa |= (B.FLAG_GATE_EXPERT if args.smha_mode != "data" else 0) | (B.FLAG_GATE_PATCH if args.smha_mode != "expert" else 0)
    fm = B.FLAG_RESIDUAL | B.FLAG_GATE_EXPERT | (B.FLAG_GATE_PATCH if uome_ds else 0)
    dev = DeviceLayer(inp, fa, fm, device="cuda:0", rope_dim=args.rope_dim)
    torch.cuda.set_device(0)

    if args.stage:
        return run_stage(args, cfg, dev, B, torch,
                         lambda: DeviceLayer(inp, fa, fm, device="cuda:0", rope_dim=args.rope_dim))

    # ---- whole-path throughput.  The layer call only enqueues kernels (no allocation, no memset, no
    # synchronisation), so it can also be captured into a HIP graph (--graph: a step is one replay).
    # Either way every kernel of the path runs in every step.
    def timed(step):
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    step_fn = dev.layer_forward
    if args.dynamic_capacity:
        import dataclasses
        cap = torch.zeros((cfg.b,), dtype=torch.int32, device=dev.device)
        by_c = {}

        def dynamic_step():
            B.route_capacity(dev.smha, dev.x, dev.a_w_b, dev.a_w_a, dev.noise_a_patch, args.dynamic_capacity, cap, None,
                             None, dev.ws)
            c_dyn = int(cap.max().item())          # the host needs c to size the call: one read-back per step
            if c_dyn not in by_c:                  # same inputs, another descriptor / buffers for this c
                by_c[c_dyn] = DeviceLayer(dataclasses.replace(inp, cfg=dataclasses.replace(cfg, c=c_dyn)), fa, fm,
                                          device="cuda:0", rope_dim=args.rope_dim)
            by_c[c_dyn].layer_forward()
        dynamic_step()
        cfg = next(iter(by_c.values())).cfg        # report the shape that actually ran
        step_fn = dynamic_step
    eager_ms = timed(step_fn)
    launch = "eager"
    ms_per_step = eager_ms
    n_streams = 1 if (args.graph or args.dynamic_capacity) else max(1, args.streams)
    if n_streams > 1:
        # S replicas of the layer's buffers (same synthetic batch, separate allocations), one stream each
        lanes = [dev] + [DeviceLayer(inp, fa, fm, device="cuda:0", rope_dim=args.rope_dim) for _ in range(n_streams - 1)]
        # lane 0 stays on the stream everything so far ran on (it already owns a hardware queue)
        streams = [torch.cuda.current_stream()] + [torch.cuda.Stream() for _ in lanes[1:]]
        raw = [int(st.cuda_stream) for st in streams]   # the hipStream_t values the C ABI takes
        torch.cuda.synchronize()                        # the replicas' uploads ran on the default stream

        def timed_lanes():
            def run(count):
                for i in range(count):
                    lanes[i % n_streams].layer_forward(stream=raw[i % n_streams])
            run(max(args.warmup, n_streams))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            run(args.steps)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / args.steps
        ms_per_step = timed_lanes()
        launch = f"eager, {n_streams} streams (independent steps in flight)"
        for lane in lanes[1:]:   # every lane ran the same batch through the same kernels
            if not torch.equal(lane.out, dev.out):
                print("bench.py: lanes disagree", file=sys.stderr)
                return 1
        del lanes[1:]
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            dev.layer_forward()
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            dev.layer_forward()
        ms_per_step = timed(graph.replay)
        launch = "hip graph replay"
    tokens_per_s = cfg.tokens / (ms_per_step * 1e-3)
    fl = layer_flops(cfg)

    # ---- dominant kernel: the UoME up-projection grouped GEMM (half of the UoME FLOPs, which are
    # 84-90% of the layer).  Timed alone with events on the stream it is launched on.
    hidden = torch.empty((cfg.b, cfg.l, cfg.k_m * cfg.d_e), dtype=dev.tdtype, device=dev.device)
    up = lambda: B.uome_up(dev.uome, dev.u, dev.a_in, dev.m_expert_idx, dev.m_expert_gate, hidden)
    dev.smha_forward()          # u, then the UoME routing the GEMM reads
    dev.route_m()
    if uome_ds:                 # no separate entry point for the first layer: time the block's two GEMMs together
        up = dev.uome_forward
    for _ in range(max(3, args.warmup)):
        up()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    src = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev.device).zero_()
    dst = torch.empty_like(src)

    def gpu_paced(fn, count):
        """Mean time of `count` launches of fn on the current stream, by events, with the launches queued
        while the GPU is still busy with large copies: what is timed is the GPU working through its queue,
        not the host filling it.  Second value: whether the host really stayed ahead."""
        torch.cuda.synchronize()
        for _ in range(8):
            dst.copy_(src)
        ev0.record()
        for _ in range(count):
            fn()
        ev1.record()
        ahead = not ev0.query()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / count, ahead
    up_launches = min(args.steps, 200)
    up_ms, up_ahead = gpu_paced(up, up_launches)
    up_flops = float(fl["uome"]) if uome_ds else 2.0 * cfg.b * cfg.l * cfg.d * cfg.k_m * cfg.d_e
    is_bf16 = cfg.dtype == synth.BF16
    peak = PEAK_BF16_TFLOPS if is_bf16 else PEAK_FP32_TFLOPS
    achieved = up_flops / (up_ms * 1e-3) / 1e12
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath) and not uome_ds:
        traffic = json.load(open(tpath)).get(f"uome_up:{cfg.name}")
    roofline = {"kernel": "uome_forward, data selection (Eq. 37-40: both grouped GEMMs)" if uome_ds
                else "uome_up (Eq. 38 grouped GEMM + SiLU + gate)", "bound": "mfma",
                "achieved": round(achieved, 3), "peak": peak, "unit": "TFLOP/s",
                "frac": round(achieved / peak, 5), "traffic": traffic,
                "flops_per_launch": up_flops, "ms_per_launch": round(up_ms, 5), "launches_timed": up_launches,
                "host_stayed_ahead": up_ahead}

    # ---- what a dependent launch costs on the GPU's side whatever the kernel does: the smallest kernel of
    # the library (the gather of the 128-token fp32 shape) 100 times on one stream, queued while the GPU is
    # still busy (gpu_paced above; the figure is dropped if the GPU caught up with the host before
    # everything was queued).  Context for the small shapes: their
    # kernels take several times this, they are chains of dependent memory round trips in a single round
    # of workgroups, which is why independent steps in flight fill the GPU.
    tiny_inp = synth.make_inputs(synth.CONFIGS["tiny"])
    tiny_inp.noise_m_patch = None
    tiny = DeviceLayer(tiny_inp, B.FLAG_RESIDUAL, B.FLAG_RESIDUAL, device="cuda:0")
    tiny.layer_forward()
    tcfg = tiny.cfg
    th = torch.empty((tcfg.b, tcfg.k_a, tcfg.l_a, tcfg.d), dtype=tiny.tdtype, device=tiny.device)
    small = lambda: B.gather(tiny.smha, tiny.x, tiny.a_expert_idx, tiny.a_patch_idx, th)
    for _ in range(10):
        small()
    floor_ms, floor_ahead = gpu_paced(small, 100)
    roofline["dependent_launch_floor_us"] = round(floor_ms * 1e3, 2) if floor_ahead else None
    del src, dst

    # ---- CPU oracle on this machine's host cores, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        nb = cfg.b
        # keep the sample to a few GFLOP-fp64-seconds: whole batch for the small shapes, else 1 sample
        if fl["total"] > 4e10:
            nb = 1

        class _Sub:   # the first nb samples of the same inputs
            pass
        sub = _Sub()
        sub.__dict__.update(inp.__dict__)
        sub.x = inp.x[:nb]
        for f in ("noise_a_expert", "noise_a_patch", "noise_m_expert"):
            v = getattr(inp, f)
            setattr(sub, f, None if v is None else v[:nb])
        oracle.layer_forward(sub, fa, fm, args.rope_dim) if fl["total"] * nb / cfg.b < 2e10 else None   # warm the pages
        passes = 0
        c0 = time.perf_counter()
        while True:   # whole passes until about 10 s of CPU work have been timed
            oracle.layer_forward(sub, fa, fm, args.rope_dim)
            passes += 1
            c1 = time.perf_counter()
            if c1 - c0 >= 10.0 or passes >= 400:
                break
        cpu = {"value": round(passes * nb * cfg.l / (c1 - c0), 1), "unit": "tokens/s", "cores": oracle.get_threads(),
               "kind": "oracle", "sample": f"{nb} of {cfg.b} samples of the {cfg.name} workload, {passes} fp64 "
                                           f"pass(es) in {c1 - c0:.2f} s"}

    line = {
        "metric": "UoE layer fwd tokens/sec (SMHA+UoME) at 1 GPU",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if is_bf16 else "f32", "data": "synthetic",
        "config": {"workload": describe(cfg),
                   "flags": "residual" + ("+expert gate" if fa & B.FLAG_GATE_EXPERT else "") +
                            ("+patch gate" if fa & B.FLAG_GATE_PATCH else "") + ("+causal" if args.causal else "") +
                            (f"+rope{args.rope_dim}" if args.rope_dim else "") +
                            (f"; SMHA {args.smha_mode} selection only" if args.smha_mode != "both" else "") +
                            ("; UoME data selection, +patch gate" if uome_ds else "") +
                            (f"; SMHA c from Eq. 15-16 with {args.dynamic_capacity} experts per patch, read back every step"
                             if args.dynamic_capacity else ""),
                   "seed": cfg.seed, "launch": launch},
        "single_stream": {"ms_per_step": round(eager_ms, 5), "value": round(cfg.tokens / (eager_ms * 1e-3), 1)},
        "tflops": round(fl["total"] / (ms_per_step * 1e-3) / 1e12, 3),
        "flops_per_step": fl["total"],
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
