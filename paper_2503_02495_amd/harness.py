"""Device-side plumbing for tests and the benchmark: upload a synthetic input set, allocate
outputs and workspace with torch, and call the C ABI through ``binding``.  No arithmetic."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as B
from . import synth


def to_device(a: Optional[np.ndarray], dtype: str, device) -> Optional[torch.Tensor]:
    """float32 host array -> device tensor of the storage dtype (bf16 values must be bf16-exact)."""
    if a is None:
        return None
    if dtype == synth.BF16:
        bits = synth.bf16_bits(a)
        return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    """device tensor -> float64 / int32 host array."""
    if t.dtype in (torch.int32, torch.int64):
        return t.cpu().numpy().astype(np.int32)
    return t.to(torch.float32).cpu().numpy().astype(np.float64)


class DeviceLayer:
    """One UoE layer's tensors resident on the GPU, plus descriptors, outputs and workspace."""

    def __init__(self, inp: synth.LayerInputs, flags_a: int, flags_m: int, device="cuda:0", rope_dim: int = 0):
        cfg = inp.cfg
        self.cfg, self.device = cfg, torch.device(device)
        dt = cfg.dtype
        self.tdtype = torch.bfloat16 if dt == synth.BF16 else torch.float32
        code = B.BF16 if dt == synth.BF16 else B.F32
        up = lambda a: to_device(a, dt, self.device)
        f32 = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(self.device)
        self.x = up(inp.x)
        self.a_w_expert, self.a_w_b, self.a_w_a = up(inp.a_w_expert), up(inp.a_w_b), up(inp.a_w_a)
        self.wq, self.wk, self.wv, self.wo = up(inp.wq), up(inp.wk), up(inp.wv), up(inp.wo)
        self.m_w_expert, self.a_in, self.a_out = up(inp.m_w_expert), up(inp.a_in), up(inp.a_out)
        self.noise_a_expert, self.noise_a_patch = f32(inp.noise_a_expert), f32(inp.noise_a_patch)
        self.noise_m_expert = f32(inp.noise_m_expert)
        self.m_w_b, self.m_w_a = up(getattr(inp, "m_w_b", None)), up(getattr(inp, "m_w_a", None))
        self.noise_m_patch = f32(getattr(inp, "noise_m_patch", None))
        self.uome_ds = cfg.m_m > 1

        self.smha = B.block_desc(cfg.b, cfg.l, cfg.d, cfg.n_a, cfg.k_a, cfg.m, cfg.c, cfg.d_h, code, flags_a, rope_dim)
        self.uome = B.block_desc(cfg.b, cfg.l, cfg.d, cfg.n_m, cfg.k_m, cfg.m_m, cfg.c_m, cfg.d_e, code, flags_m)
        nbytes = B.workspace_bytes(self.smha, self.uome)
        if nbytes == 0:
            raise B.UoeError(B.ERR_INVALID_ARG, "uoe_workspace_bytes")
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)

        i32 = dict(dtype=torch.int32, device=self.device)
        f = dict(dtype=torch.float32, device=self.device)
        self.a_expert_idx = torch.full((cfg.b, cfg.k_a), -1, **i32)
        self.a_expert_gate = torch.zeros((cfg.b, cfg.n_a), **f)
        self.a_patch_idx = torch.full((cfg.b, cfg.n_a, cfg.c), -1, **i32)
        self.a_patch_gate = torch.zeros((cfg.b, cfg.n_a, cfg.m), **f)
        self.m_expert_idx = torch.full((cfg.b, cfg.k_m), -1, **i32)
        self.m_expert_gate = torch.zeros((cfg.b, cfg.n_m), **f)
        self.m_patch_idx = torch.full((cfg.b, cfg.n_m, cfg.c_m), -1, **i32) if self.uome_ds else None
        self.m_patch_gate = torch.zeros((cfg.b, cfg.n_m, cfg.m_m), **f) if self.uome_ds else None
        self.u = torch.zeros((cfg.b, cfg.l, cfg.d), dtype=self.tdtype, device=self.device)
        self.out = torch.zeros((cfg.b, cfg.l, cfg.d), dtype=self.tdtype, device=self.device)
        self.wa = B.smha_weights(self.a_w_expert, self.a_w_b, self.a_w_a, self.wq, self.wk, self.wv, self.wo)
        self.wm = B.uome_weights(self.m_w_expert, self.a_in, self.a_out, self.m_w_b, self.m_w_a)
        self.ra = B.routing_out(self.a_expert_idx, self.a_expert_gate, self.a_patch_idx, self.a_patch_gate)
        self.rm = B.routing_out(self.m_expert_idx, self.m_expert_gate, self.m_patch_idx, self.m_patch_gate)

    # each method is one C-ABI call on the current stream
    def route_a(self):
        B.route(self.smha, self.x, self.a_w_expert, self.a_w_b, self.a_w_a, self.noise_a_expert,
                self.noise_a_patch, self.a_expert_idx, self.a_expert_gate, self.a_patch_idx,
                self.a_patch_gate, self.ws)

    def smha_forward(self, expert_idx=None, expert_gate=None, patch_idx=None, patch_gate=None, x=None, out=None,
                     pad_mask=None):
        args = (self.smha, self.x if x is None else x, self.wq, self.wk, self.wv, self.wo,
                self.a_expert_idx if expert_idx is None else expert_idx,
                self.a_expert_gate if expert_gate is None else expert_gate,
                self.a_patch_idx if patch_idx is None else patch_idx,
                self.a_patch_gate if patch_gate is None else patch_gate)
        if pad_mask is None:
            B.smha_forward(*args, self.u if out is None else out, self.ws)
        else:
            B.smha_forward_masked(*args, pad_mask, self.u if out is None else out, self.ws)

    def route_m(self, u=None):
        B.route(self.uome, self.u if u is None else u, self.m_w_expert, self.m_w_b, self.m_w_a, self.noise_m_expert,
                self.noise_m_patch, self.m_expert_idx, self.m_expert_gate, self.m_patch_idx, self.m_patch_gate, self.ws)

    def uome_forward(self, expert_idx=None, expert_gate=None, u=None, out=None, patch_idx=None, patch_gate=None):
        if self.uome_ds and patch_idx is None:
            patch_idx, patch_gate = self.m_patch_idx, self.m_patch_gate
        B.uome_forward(self.uome, self.u if u is None else u, self.a_in, self.a_out,
                       self.m_expert_idx if expert_idx is None else expert_idx,
                       self.m_expert_gate if expert_gate is None else expert_gate, patch_idx, patch_gate,
                       self.out if out is None else out, self.ws)

    def uome_backward(self, d_out, expert_idx=None, expert_gate=None, u=None, patch_idx=None, patch_gate=None):
        """Gradients of the UoME block; returns (d_u, d_a_in, d_a_out, d_gate) and, for a data-selection
        block, d_patch_gate as a fifth member."""
        if self.uome_ds and patch_idx is None:
            patch_idx, patch_gate = self.m_patch_idx, self.m_patch_gate
        if not hasattr(self, "bwd_ws"):
            nbytes = B.uome_backward_workspace_bytes(self.uome)
            if nbytes == 0:
                raise B.UoeError(B.ERR_UNSUPPORTED, "uoe_uome_backward_workspace_bytes")
            self.bwd_ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self.d_u = torch.empty_like(self.x)
            self.d_a_in, self.d_a_out = torch.empty_like(self.a_in), torch.empty_like(self.a_out)
            self.d_gate = torch.empty(self.cfg.b, self.cfg.n_m, dtype=torch.float32, device=self.device)
            self.d_m_patch_gate = (torch.empty(self.cfg.b, self.cfg.n_m, self.cfg.m_m, dtype=torch.float32, device=self.device)
                                   if self.uome_ds else None)
        B.uome_backward(self.uome, self.u if u is None else u, self.a_in, self.a_out,
                        self.m_expert_idx if expert_idx is None else expert_idx,
                        self.m_expert_gate if expert_gate is None else expert_gate, patch_idx, patch_gate, d_out,
                        self.d_u, self.d_a_in, self.d_a_out, self.d_gate, self.d_m_patch_gate, self.bwd_ws)
        if self.uome_ds:
            return self.d_u, self.d_a_in, self.d_a_out, self.d_gate, self.d_m_patch_gate
        return self.d_u, self.d_a_in, self.d_a_out, self.d_gate

    def smha_backward(self, d_out, expert_idx=None, expert_gate=None, patch_idx=None, patch_gate=None, pad_mask=None):
        """Gradients of the SMHA block; returns (d_x, d_wq, d_wk, d_wv, d_wo, d_expert_gate, d_patch_gate)."""
        if not hasattr(self, "smha_bwd_ws"):
            nbytes = B.smha_backward_workspace_bytes(self.smha)
            if nbytes == 0:
                raise B.UoeError(B.ERR_UNSUPPORTED, "uoe_smha_backward_workspace_bytes")
            self.smha_bwd_ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self.d_x = torch.empty_like(self.x)
            self.d_wq, self.d_wk, self.d_wv = (torch.empty_like(t) for t in (self.wq, self.wk, self.wv))
            self.d_wo = torch.empty_like(self.wo)
            cfg = self.cfg
            self.d_a_expert_gate = torch.empty(cfg.b, cfg.n_a, dtype=torch.float32, device=self.device)
            self.d_a_patch_gate = torch.empty(cfg.b, cfg.n_a, cfg.m, dtype=torch.float32, device=self.device)
            self.smha_dw = B.smha_weight_grads(self.d_wq, self.d_wk, self.d_wv, self.d_wo)
        B.smha_backward(self.smha, self.x, self.wa,
                        self.a_expert_idx if expert_idx is None else expert_idx,
                        self.a_expert_gate if expert_gate is None else expert_gate,
                        self.a_patch_idx if patch_idx is None else patch_idx,
                        self.a_patch_gate if patch_gate is None else patch_gate, pad_mask, d_out, self.d_x, self.smha_dw,
                        self.d_a_expert_gate, self.d_a_patch_gate, self.smha_bwd_ws)
        return self.d_x, self.d_wq, self.d_wk, self.d_wv, self.d_wo, self.d_a_expert_gate, self.d_a_patch_gate

    def layer_backward(self, d_out, routing_a=None, routing_m=None, u=None, pad_mask=None, stream=None):
        """Gradients of the whole layer for d_out = dL/d(out).  routing_a / routing_m default to the
        results the last layer_forward wrote; u = None has it recomputed; pad_mask as in the forward
        call.  Returns a dict of tensors."""
        if not hasattr(self, "layer_bwd_ws"):
            nbytes = B.layer_backward_workspace_bytes(self.smha, self.uome)
            if nbytes == 0:
                raise B.UoeError(B.ERR_UNSUPPORTED, "uoe_layer_backward_workspace_bytes")
            self.layer_bwd_ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            like = lambda t: None if t is None else torch.empty_like(t)
            self.g = {"d_x": like(self.x), "d_wq": like(self.wq), "d_wk": like(self.wk), "d_wv": like(self.wv),
                      "d_wo": like(self.wo), "d_a_w_expert": like(self.a_w_expert), "d_a_w_b": like(self.a_w_b),
                      "d_a_w_a": like(self.a_w_a), "d_a_in": like(self.a_in), "d_a_out": like(self.a_out),
                      "d_m_w_expert": like(self.m_w_expert), "d_m_w_b": like(self.m_w_b), "d_m_w_a": like(self.m_w_a)}
            g = self.g
            self.layer_dwa = B.smha_weight_grads(g["d_wq"], g["d_wk"], g["d_wv"], g["d_wo"])
            self.layer_dra = B.router_grads(g["d_a_w_expert"], g["d_a_w_b"], g["d_a_w_a"])
            self.layer_drm = B.router_grads(g["d_m_w_expert"], g["d_m_w_b"], g["d_m_w_a"])
        tail = (self.ra if routing_a is None else routing_a, self.rm if routing_m is None else routing_m, d_out,
                self.g["d_x"], self.layer_dwa, self.layer_dra, self.g["d_a_in"], self.g["d_a_out"], self.layer_drm,
                self.layer_bwd_ws)
        if pad_mask is None:
            B.layer_backward(self.smha, self.wa, self.uome, self.wm, self.x, u, *tail, stream=stream)
        else:
            B.layer_backward_masked(self.smha, self.wa, self.uome, self.wm, self.x, pad_mask, u, *tail, stream=stream)
        return self.g

    def layer_forward(self, pad_mask=None, stream=None):
        """stream: a torch stream or a raw hipStream_t value; None = torch's current stream."""
        if pad_mask is None:
            B.layer_forward(self.smha, self.wa, self.noise_a_expert, self.noise_a_patch, self.uome, self.wm,
                            self.noise_m_expert, self.x, self.out, self.ra, self.rm, self.ws, stream=stream)
        else:
            B.layer_forward_masked(self.smha, self.wa, self.noise_a_expert, self.noise_a_patch, self.uome, self.wm,
                                   self.noise_m_expert, self.x, pad_mask, self.out, self.ra, self.rm, self.ws, stream=stream)
