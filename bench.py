#!/usr/bin/env python3
"""Throughput of one Union-of-Experts layer forward (uoe_layer_forward) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large|lm|longrange|vit|tiny]

A step is one pass of the whole hot path (route -> SMHA -> route -> UoME) over one batch of seeded
synthetic input that is already resident in HBM; steps run one after the other on one stream.
After W warm-up steps, K steps are timed between two synchronisations with events on the launch
stream; that region is repeated (--regions) and the median region is reported.  Prints ONE JSON
line: whole-job tokens/s, a roofline entry for the dominant kernel and one per kernel of the layer
(each timed live with events on the launch stream against its algorithmic FLOPs or bytes), what
the device delivers for a plain copy / read-only stream / MFMA loop, the realised expert loads,
and the CPU oracle timed on this machine's host cores as a reported baseline (with the selection
parity and near-tie counts of the timed batch).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
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


def kernel_work(c, es: int) -> dict:
    """Algorithmic work of each kernel of the layer call: FLOPs and the HBM bytes the method itself
    has to move (every operand once, active units only), per launch.  es = bytes per stored element."""
    bld = c.b * c.l * c.d
    units_a = c.b * c.k_a
    hidden = c.b * c.l * c.k_m * c.d_e
    return {
        # Eq. 21: x and W_E once each
        "route_expert_a": dict(eq="Eq. 21-22", flops=2 * bld * c.n_a, bytes=(bld + c.n_a * c.l * c.d) * es),
        # Eq. 13-14, 17: x once, W_B, W_A
        "route_data_a": dict(eq="Eq. 13-14, 17", flops=2 * bld * c.n_a + 2 * c.b * c.n_a * c.l * c.m,
                             bytes=(bld + c.d * c.n_a + c.l * c.m) * es),
        # both SMHA routers read the same x: once
        "route_a": dict(eq="Eq. 13-14, 17, 21-22", flops=4 * bld * c.n_a + 2 * c.b * c.n_a * c.l * c.m,
                        bytes=(bld + c.n_a * c.l * c.d + c.d * c.n_a + c.l * c.m) * es),
        "gather": dict(eq="Eq. 18", flops=0, bytes=2 * units_a * c.l_a * c.d * es),
        # gathered rows in, q/k/v out, the active experts' projection weights
        "smha_qkv": dict(eq="Eq. 18, 28-30", flops=6 * units_a * c.l_a * c.d * c.d_h,
                         bytes=(units_a * c.l_a * c.d + 3 * units_a * c.l_a * c.d_h + 3 * c.n_a * c.d * c.d_h) * es),
        "smha_attention": dict(eq="Eq. 33-34", flops=4 * units_a * c.l_a * c.l_a * c.d_h,
                               bytes=4 * units_a * c.l_a * c.d_h * es),
        # attention output in, residual in, u out, W^o
        "smha_out": dict(eq="Eq. 35-36", flops=2 * units_a * c.l_a * c.d_h * c.d,
                         bytes=(units_a * c.l_a * c.d_h + 2 * bld + c.n_a * c.d_h * c.d) * es),
        "route_m": dict(eq="Eq. 21-22 on u", flops=2 * bld * c.n_m, bytes=(bld + c.n_m * c.l * c.d) * es),
        "uome_up": dict(eq="Eq. 38", flops=2 * bld * c.k_m * c.d_e, bytes=(bld + c.n_m * c.d * c.d_e + hidden) * es),
        "uome_down": dict(eq="Eq. 39-40", flops=2 * bld * c.k_m * c.d_e,
                          bytes=(hidden + c.n_m * c.d_e * c.d + 2 * bld) * es),
    }


def describe(c) -> str:
    ds = f" m{c.m_m} c{c.c_m}" if c.m_m > 1 else ""
    return (f"{c.name}: b{c.b} l{c.l} d{c.d}; SMHA n{c.n_a} d_h{c.d_h} m{c.m} c{c.c} k{c.k_a}; "
            f"UoME n{c.n_m} d_e{c.d_e} k{c.k_m}{ds}; {c.dtype}")


class Pacer:
    """Times launches by events with the host out of the picture: the launches are queued while the
    GPU is still busy with a few large copies (the library's own copy probe), so what is timed is the
    GPU working through its queue, not the host filling it."""

    def __init__(self, torch, B, device):
        self.torch, self.B = torch, B
        self.src = torch.zeros(1 << 28, dtype=torch.uint8, device=device)
        self.dst = torch.empty_like(self.src)
        self.ev0, self.ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def __call__(self, fn, count):
        """(mean ms per launch, whether the host stayed ahead of the GPU)."""
        torch = self.torch
        torch.cuda.synchronize()
        for _ in range(6):
            self.B.probe_copy(self.src, self.dst, self.src.numel())
        self.ev0.record()
        for _ in range(count):
            fn()
        self.ev1.record()
        ahead = not self.ev0.query()
        torch.cuda.synchronize()
        return self.ev0.elapsed_time(self.ev1) / count, ahead


def stage_calls(cfg, dev, B, torch):
    """One C-ABI call per kernel (or kernel group) of the layer, on the tensors a layer call left."""
    dev.layer_forward()      # fills routing results
    dev.smha_forward()       # u and the SMHA workspace (q, k, v, o)
    dev.route_m()
    hidden = torch.empty((cfg.b, cfg.l, cfg.k_m * cfg.d_e), dtype=dev.tdtype, device=dev.device)
    h = torch.empty((cfg.b, cfg.k_a, cfg.l_a, cfg.d), dtype=dev.tdtype, device=dev.device)
    if cfg.m_m == 1:
        B.uome_up(dev.uome, dev.u, dev.a_in, dev.m_expert_idx, dev.m_expert_gate, hidden)
    dev.smha_forward()       # again: the routing call above used the head of the workspace as its scratch
    code = dev.smha.dtype
    # single-router descriptors of the SMHA block: expert router alone (one patch), data router alone (k = n)
    blk_e = B.block_desc(cfg.b, cfg.l, cfg.d, cfg.n_a, cfg.k_a, 1, 1, cfg.d_h, code, 0)
    blk_d = B.block_desc(cfg.b, cfg.l, cfg.d, cfg.n_a, cfg.n_a, cfg.m, cfg.c, cfg.d_h, code, 0)
    i32 = dict(dtype=torch.int32, device=dev.device)
    e_idx_all = torch.empty((cfg.b, cfg.n_a), **i32)
    e_idx, e_gate = torch.empty_like(dev.a_expert_idx), torch.empty_like(dev.a_expert_gate)
    p_idx, p_gate = torch.empty_like(dev.a_patch_idx), torch.empty_like(dev.a_patch_gate)

    def smha_step(steps):
        return lambda: B.smha_forward_steps(dev.smha, dev.x, dev.wq, dev.wk, dev.wv, dev.wo, dev.a_expert_idx,
                                            dev.a_expert_gate, dev.a_patch_idx, dev.a_patch_gate, None, dev.u, dev.ws,
                                            steps)
    calls = {
        "route_a": dev.route_a, "smha": dev.smha_forward, "route_m": dev.route_m, "uome": dev.uome_forward,
        "route_expert_a": (lambda: B.route(blk_e, dev.x, dev.a_w_expert, None, None, dev.noise_a_expert, None, e_idx, e_gate,
                                           None, None, dev.ws)) if dev.a_w_expert is not None else None,
        "route_data_a": (lambda: B.route(blk_d, dev.x, None, dev.a_w_b, dev.a_w_a, None, dev.noise_a_patch, e_idx_all, None,
                                         p_idx, p_gate, dev.ws)) if dev.a_w_b is not None else None,
        "smha_qkv": smha_step(B.SMHA_STEP_QKV), "smha_attention": smha_step(B.SMHA_STEP_ATTENTION),
        "smha_out": smha_step(B.SMHA_STEP_OUT),
        "uome_up": (lambda: B.uome_up(dev.uome, dev.u, dev.a_in, dev.m_expert_idx, dev.m_expert_gate, hidden))
        if cfg.m_m == 1 else None,
        "uome_down": (lambda: B.uome_down(dev.uome, hidden, dev.a_out, dev.u, dev.m_expert_idx, dev.out))
        if cfg.m_m == 1 else None,
        "gather": lambda: B.gather(dev.smha, dev.x, dev.a_expert_idx, dev.a_patch_idx, h),
    }
    return {k: v for k, v in calls.items() if v is not None}


def run_stage(args, cfg, dev, B, torch, make_lane) -> int:
    """Loop one stage (its inputs produced once by the stages before it) and print its mean time."""
    calls = stage_calls(cfg, dev, B, torch)
    if args.stage in ("probe_copy", "probe_read"):   # transfers of known size (1 GiB): counter calibration
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev.device).random_(0, 255)
        dst = torch.empty_like(src)
        sink = torch.empty(4096, dtype=torch.int32, device=dev.device)
        calls["probe_copy"] = lambda: B.probe_copy(src, dst, src.numel())
        calls["probe_read"] = lambda: B.probe_read(src, src.numel(), sink)
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
    if args.stage == "layer_fwd_bwd" and args.stage_streams > 1:
        # a training step per batch, several independent batches in flight (one lane per stream, lane 0 on the
        # program's own stream)
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
    if args.stage not in calls:
        print(f"bench.py: stage {args.stage} does not apply to this configuration", file=sys.stderr)
        return 2
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


def measured_ceilings(B, torch, device, pace) -> dict:
    """What this device delivers for a plain copy, a read-only stream and a register-resident bf16 MFMA
    loop (the library's probe kernels): the scale next to the published peaks."""
    import numpy as np
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=device).random_(0, 255)
    dst = torch.empty_like(src)
    sink = torch.empty(4096, dtype=torch.int32, device=device)
    out = {}
    for _ in range(2):
        B.probe_copy(src, dst, n)
        B.probe_read(src, n, sink)
    ms, _ = pace(lambda: B.probe_copy(src, dst, n), 10)
    out["copy_GBs"] = round(2.0 * n / (ms * 1e-3) / 1e9, 1)          # bytes read + bytes written
    ms, _ = pace(lambda: B.probe_read(src, n, sink), 10)
    out["read_GBs"] = round(n / (ms * 1e-3) / 1e9, 1)
    del src, dst
    msink = torch.empty(131072, dtype=torch.float32, device=device)
    rng = np.random.default_rng(0)
    vals = rng.standard_normal(6 * 64 * 8).astype(np.float32)
    for tag, host in (("zeros", np.zeros_like(vals)), ("random", vals)):
        ops = torch.from_numpy(host).to(device).to(torch.bfloat16).contiguous()
        iters = 20000
        B.probe_mfma(ops, iters, msink)
        flops = [0.0]

        def run():
            flops[0] = B.probe_mfma(ops, iters, msink)
        ms, _ = pace(run, 5)
        out[f"mfma_bf16_TFLOPs_{tag}_operands"] = round(flops[0] / (ms * 1e-3) / 1e12, 1)
    out["note"] = ("library probe kernels on this device: 1 GiB copy (read + write bytes counted), 1 GiB read-only "
                   "stream, MFMA 32x32x16 bf16 loop without memory traffic")
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="large",
                    help="large (default: the largest single-GPU shape), lm, longrange, vit or tiny")
    ap.add_argument("--regions", type=int, default=5,
                    help="how many times the timed region of --steps steps is repeated; the median region is reported")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-rooflines", action="store_true", help="skip the per-kernel timings and the probes")
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
    ap.add_argument("--streams", type=int, default=1, metavar="S",
                    help="S > 1: additionally report (extra key steps_in_flight) the rate with S independent steps in "
                         "flight, step i on HIP stream i %% S with its own inputs, workspace and output.  The headline "
                         "value is always one call after the other on one stream")
    ap.add_argument("--stage-streams", type=int, default=1, metavar="S",
                    help="with --stage layer_fwd_bwd: S independent training steps in flight, one lane per stream")
    ap.add_argument("--stage", default=None,
                    choices=["route_a", "route_expert_a", "route_data_a", "smha", "smha_qkv", "smha_attention", "smha_out",
                             "route_m", "uome", "uome_up", "uome_down", "gather", "probe_copy", "probe_read",
                             "uome_bwd", "smha_bwd", "route_bwd", "layer_bwd", "layer_fwd_bwd"],
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
    from paper_2503_02495_amd.harness import DeviceLayer, to_host

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

    # ---- whole-path throughput: one layer call after the other on one stream.  The call only enqueues
    # kernels (no allocation, no memset, no synchronisation); every kernel of the path runs in every step.
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

    for _ in range(args.warmup):
        step_fn()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    region_ms, region_wall_ms = [], []
    for _ in range(max(1, args.regions)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for _ in range(args.steps):
            step_fn()
        ev1.record()
        torch.cuda.synchronize()
        region_wall_ms.append((time.perf_counter() - t0) * 1e3 / args.steps)
        region_ms.append(ev0.elapsed_time(ev1) / args.steps)
    ms_per_step = statistics.median(region_ms)
    tokens_per_s = cfg.tokens / (ms_per_step * 1e-3)
    fl = layer_flops(cfg)
    is_bf16 = cfg.dtype == synth.BF16
    es = 2 if is_bf16 else 4
    peak_tf = PEAK_BF16_TFLOPS if is_bf16 else PEAK_FP32_TFLOPS

    # ---- independent steps in flight (extra key only)
    in_flight = None
    if args.streams > 1 and not args.dynamic_capacity:
        n_streams = args.streams
        lanes = [dev] + [DeviceLayer(inp, fa, fm, device="cuda:0", rope_dim=args.rope_dim) for _ in range(n_streams - 1)]
        streams = [torch.cuda.current_stream()] + [torch.cuda.Stream() for _ in lanes[1:]]
        raw = [int(st.cuda_stream) for st in streams]   # the hipStream_t values the C ABI takes
        torch.cuda.synchronize()                        # the replicas' uploads ran on the default stream

        def run(count):
            for i in range(count):
                lanes[i % n_streams].layer_forward(stream=raw[i % n_streams])
        run(max(args.warmup, n_streams))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(args.steps)
        torch.cuda.synchronize()
        lanes_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        for lane in lanes[1:]:   # every lane ran the same batch through the same kernels
            if not torch.equal(lane.out, dev.out):
                print("bench.py: lanes disagree", file=sys.stderr)
                return 1
        del lanes[1:]
        in_flight = {"streams": n_streams, "ms_per_step": round(lanes_ms, 5),
                     "value": round(cfg.tokens / (lanes_ms * 1e-3), 1), "clock": "host wall clock"}

    # ---- realised expert loads of the timed batch (Eq. 23: how many samples each expert serves)
    dev.layer_forward()
    torch.cuda.synchronize()
    loads = {"smha_samples_per_expert": np.bincount(to_host(dev.a_expert_idx).ravel(), minlength=cfg.n_a).tolist(),
             "uome_samples_per_expert": np.bincount(to_host(dev.m_expert_idx).ravel(), minlength=cfg.n_m).tolist()}
    pidx = to_host(dev.a_patch_idx)
    eidx = to_host(dev.a_expert_idx)
    picks = np.zeros((cfg.b, cfg.m), np.int64)       # how many active experts picked each patch
    for bb in range(cfg.b):
        for i in eidx[bb]:
            picks[bb, pidx[bb, i]] += 1
    loads["smha_patches_by_pick_count"] = np.bincount(picks.ravel(), minlength=cfg.k_a + 1).tolist()

    # ---- per-kernel rooflines: every kernel of the layer call through its own C-ABI entry point, on the
    # tensors the layer call left, timed with events on the launch stream while the host stays ahead
    kernels, ceilings, roofline = [], None, None
    if not args.no_kernel_rooflines and not uome_ds and not args.dynamic_capacity:
        pace = Pacer(torch, B, dev.device)
        calls = stage_calls(cfg, dev, B, torch)
        work = kernel_work(cfg, es)
        launches = max(5, min(args.steps, 50))
        ridge = peak_tf * 1e12 / (PEAK_HBM_GBS * 1e9)
        # HBM-side bytes per launch measured with hardware counters (profiles/traffic.json, written from the
        # rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summaries beside it), where a summary covers the kernel
        tpath = os.path.join(ROOT, "profiles", "traffic.json")
        measured_traffic = json.load(open(tpath)) if os.path.exists(tpath) else {}
        for name in ("route_expert_a", "route_data_a", "route_a", "gather", "smha_qkv", "smha_attention", "smha_out",
                     "route_m", "uome_up", "uome_down"):
            if name not in calls:
                continue
            fn, w = calls[name], work[name]
            for _ in range(3):
                fn()
            ms, ahead = pace(fn, launches)
            gbs, tfs = w["bytes"] / (ms * 1e-3) / 1e9, w["flops"] / (ms * 1e-3) / 1e12
            bound = "mfma" if is_bf16 and w["bytes"] and w["flops"] / w["bytes"] >= ridge else "hbm"
            if not is_bf16 and w["flops"] / max(w["bytes"], 1) >= PEAK_FP32_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
                bound = "alu"
            ach, peak, unit = (gbs, PEAK_HBM_GBS, "GB/s") if bound == "hbm" else (tfs, peak_tf, "TFLOP/s")
            kernels.append({"kernel": name, "eq": w["eq"], "bound": bound, "achieved": round(ach, 2), "peak": peak,
                            "unit": unit, "frac": round(ach / peak, 4), "us_per_launch": round(ms * 1e3, 2),
                            "flops": w["flops"], "bytes": w["bytes"], "GBs": round(gbs, 1), "TFLOPs": round(tfs, 2),
                            "launches_timed": launches, "host_stayed_ahead": ahead,
                            "traffic": measured_traffic.get(f"{name}:{cfg.name}"),
                            "note": {"route_expert_a": "expert router + its selection kernel",
                                     "route_data_a": "data router + reduction + selection kernels",
                                     "route_a": "the whole SMHA routing call (both routers, selection)",
                                     "route_m": "UoME expert router + its selection kernel",
                                     "gather": "standalone Eq. 18 copy; the layer call folds it into smha_qkv"}.get(name)})
        # the dominant kernel: the single-kernel stage that takes the most time
        single = [k for k in kernels if k["kernel"] not in ("route_a", "gather")]
        dom = max(single, key=lambda k: k["us_per_launch"])
        traffic = measured_traffic.get(f"{dom['kernel']}:{cfg.name}")
        roofline = {"kernel": f"{dom['kernel']} ({dom['eq']})", "bound": dom["bound"], "achieved": dom["achieved"],
                    "peak": dom["peak"], "unit": dom["unit"], "frac": dom["frac"], "traffic": traffic,
                    "algorithmic_flops_per_launch": dom["flops"], "algorithmic_bytes_per_launch": dom["bytes"],
                    "ms_per_launch": round(dom["us_per_launch"] * 1e-3, 5), "launches_timed": launches,
                    "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary under profiles/ (bytes per launch)"
                    if traffic is not None else None}
        ceilings = measured_ceilings(B, torch, dev.device, pace)
        del pace

    # ---- CPU oracle on this machine's host cores, on a bounded sample of the same workload; with it, the
    # selection parity of the timed batch (indices bit-exact except on rows the oracle flags as near-ties)
    cpu, selection = None, None
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
        if args.smha_mode == "both" and not uome_ds and not args.dynamic_capacity:
            # routing of the whole timed batch by the oracle (routers only: a few GFLOP)
            ra = oracle.route(inp.x, cfg.n_a, cfg.k_a, cfg.m, cfg.c, inp.a_w_expert, inp.a_w_b, inp.a_w_a,
                              inp.noise_a_expert, inp.noise_a_patch)
            dev.smha_forward()
            torch.cuda.synchronize()
            rm = oracle.route(to_host(dev.u), cfg.n_m, cfg.k_m, 1, 1, inp.m_w_expert, None, None, inp.noise_m_expert, None)

            def rows(got, want, margin):
                differ = np.any(np.asarray(got) != np.asarray(want), axis=-1)
                flagged = (margin >= 0) & (margin <= oracle.NEAR_TIE_REL)
                return {"rows": int(differ.size), "near_ties": int(flagged.sum()), "mismatching_rows": int(differ.sum()),
                        "mismatching_rows_not_near_ties": int((differ & ~flagged).sum())}
            selection = {"near_tie_rel": oracle.NEAR_TIE_REL,
                         "smha_expert": rows(eidx, ra.expert_id, ra.expert_margin),
                         "smha_patch": rows(pidx, ra.patch_id, ra.patch_margin),
                         "uome_expert_on_device_u": rows(to_host(dev.m_expert_idx), rm.expert_id, rm.expert_margin)}

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
                   "seed": cfg.seed, "launch": "eager, one stream, one call after the other"},
        "timing": {"clock": "events on the launch stream around each region of `steps` calls, median region",
                   "regions": len(region_ms), "ms_per_step_by_region": [round(v, 5) for v in region_ms],
                   "host_wall_ms_per_step_by_region": [round(v, 5) for v in region_wall_ms]},
        "tflops": round(fl["total"] / (ms_per_step * 1e-3) / 1e12, 3),
        "frac_of_bf16_mfma_peak": round(fl["total"] / (ms_per_step * 1e-3) / 1e12 / peak_tf, 4),
        "flops_per_step": fl["total"],
        "roofline": roofline,
        "kernels": kernels,
        "measured_ceilings": ceilings,
        "expert_load": loads,
        "selection_parity": selection,
        "steps_in_flight": in_flight,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
