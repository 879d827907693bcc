"""ctypes binding of libuoe.so: same names as the C ABI (include/uoe.h), argument marshalling only.

Tensor arguments may be torch tensors (anything with ``data_ptr()``), raw integer device
addresses, or None.  Nothing here computes: every step of the layer runs in the library's HIP
kernels.  There is no fallback -- if the library is not built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libuoe.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_DEVICE, ERR_SCRATCH_LIMIT = 0, 1, 2, 3, 4, 5
ROUTE_STATIC_SCRATCH_BYTES = 8 * 1024 * 1024
F32, BF16 = 0, 1
FLAG_RESIDUAL, FLAG_GATE_EXPERT, FLAG_GATE_PATCH, FLAG_CAUSAL = 1, 2, 4, 8

EXPORTS = ("uoe_workspace_bytes", "uoe_status_string", "uoe_route", "uoe_route_static", "uoe_route_capacity", "uoe_balance_loss", "uoe_gather",
           "uoe_smha_forward",
           "uoe_smha_forward_masked", "uoe_smha_forward_steps", "uoe_probe_copy", "uoe_probe_read", "uoe_probe_mfma",
           "uoe_uome_forward", "uoe_uome_up", "uoe_uome_down", "uoe_layer_forward", "uoe_layer_forward_masked",
           "uoe_uome_backward_workspace_bytes", "uoe_uome_backward",
           "uoe_smha_backward_workspace_bytes", "uoe_smha_backward",
           "uoe_route_backward_workspace_bytes", "uoe_route_backward",
           "uoe_layer_backward_workspace_bytes", "uoe_layer_backward", "uoe_layer_backward_masked")


class UoeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (uoe_status {status})")


class BlockDesc(ctypes.Structure):
    _fields_ = [("b", ctypes.c_int32), ("l", ctypes.c_int32), ("d", ctypes.c_int32),
                ("n", ctypes.c_int32), ("k", ctypes.c_int32), ("m", ctypes.c_int32),
                ("c", ctypes.c_int32), ("width", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("flags", ctypes.c_uint32), ("rope_dim", ctypes.c_int32),
                ("reserved", ctypes.c_int32 * 5)]


class SmhaWeights(ctypes.Structure):
    _fields_ = [(f, ctypes.c_void_p) for f in ("w_expert", "w_b", "w_a", "wq", "wk", "wv", "wo")]


class UomeWeights(ctypes.Structure):
    _fields_ = [(f, ctypes.c_void_p) for f in ("w_expert", "w_b", "w_a", "a_in", "a_out")]


class SmhaWeightGrads(ctypes.Structure):
    _fields_ = [(f, ctypes.c_void_p) for f in ("d_wq", "d_wk", "d_wv", "d_wo")]


class RouterGrads(ctypes.Structure):
    _fields_ = [(f, ctypes.c_void_p) for f in ("d_w_expert", "d_w_b", "d_w_a")]


class RoutingOut(ctypes.Structure):
    _fields_ = [(f, ctypes.c_void_p) for f in ("expert_idx", "expert_gate", "patch_idx", "patch_gate")]


_lib = None


def lib():
    """The loaded library; raises if it has not been built (there is no CPU fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2503_02495_amd.build` "
                               "(or __graft_entry__.build()) first; there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        P, S = ctypes.c_void_p, ctypes.c_size_t
        D = ctypes.POINTER(BlockDesc)
        L.uoe_workspace_bytes.argtypes = [D, D]
        L.uoe_workspace_bytes.restype = S
        L.uoe_status_string.argtypes = [ctypes.c_int]
        L.uoe_status_string.restype = ctypes.c_char_p
        L.uoe_route.argtypes = [D] + [P] * 10 + [P, S, P]
        L.uoe_route_static.argtypes = [D] + [P] * 10 + [P]
        L.uoe_route_static.restype = ctypes.c_int
        L.uoe_route_capacity.argtypes = [D, P, P, P, P, ctypes.c_int32, P, P, P, P, S, P]
        L.uoe_balance_loss.argtypes = [D, P, P, ctypes.c_float, P, P, P]
        L.uoe_gather.argtypes = [D, P, P, P, P, P]
        L.uoe_smha_forward.argtypes = [D] + [P] * 10 + [P, S, P]
        L.uoe_smha_forward_masked.argtypes = [D] + [P] * 11 + [P, S, P]
        L.uoe_smha_forward_steps.argtypes = [D] + [P] * 11 + [P, S, ctypes.c_uint32, P]
        L.uoe_probe_copy.argtypes = [P, P, S, P]
        L.uoe_probe_read.argtypes = [P, S, P, P]
        L.uoe_probe_mfma.argtypes = [P, ctypes.c_int32, P, ctypes.POINTER(ctypes.c_double), P]
        L.uoe_uome_forward.argtypes = [D] + [P] * 8 + [P, S, P]
        L.uoe_uome_backward_workspace_bytes.argtypes = [D]
        L.uoe_uome_backward_workspace_bytes.restype = S
        L.uoe_uome_backward.argtypes = [D] + [P] * 13 + [P, S, P]
        L.uoe_smha_backward_workspace_bytes.argtypes = [D]
        L.uoe_smha_backward_workspace_bytes.restype = S
        L.uoe_smha_backward.argtypes = [D, P, ctypes.POINTER(SmhaWeights), P, P, P, P, P, P, P,
                                        ctypes.POINTER(SmhaWeightGrads), P, P, P, S, P]
        L.uoe_route_backward_workspace_bytes.argtypes = [D]
        L.uoe_route_backward_workspace_bytes.restype = S
        L.uoe_route_backward.argtypes = [D] + [P] * 12 + [P, S, P]
        L.uoe_layer_backward_workspace_bytes.argtypes = [D, D]
        L.uoe_layer_backward_workspace_bytes.restype = S
        L.uoe_layer_backward.argtypes = [D, ctypes.POINTER(SmhaWeights), D, ctypes.POINTER(UomeWeights), P, P,
                                         ctypes.POINTER(RoutingOut), ctypes.POINTER(RoutingOut), P, P,
                                         ctypes.POINTER(SmhaWeightGrads), ctypes.POINTER(RouterGrads), P, P,
                                         ctypes.POINTER(RouterGrads), P, S, P]
        L.uoe_layer_backward_masked.argtypes = [D, ctypes.POINTER(SmhaWeights), D, ctypes.POINTER(UomeWeights), P, P, P,
                                                ctypes.POINTER(RoutingOut), ctypes.POINTER(RoutingOut), P, P,
                                                ctypes.POINTER(SmhaWeightGrads), ctypes.POINTER(RouterGrads), P, P,
                                                ctypes.POINTER(RouterGrads), P, S, P]
        L.uoe_uome_up.argtypes = [D, P, P, P, P, P, P]
        L.uoe_uome_down.argtypes = [D, P, P, P, P, P, P]
        L.uoe_layer_forward.argtypes = [D, ctypes.POINTER(SmhaWeights), P, P, D, ctypes.POINTER(UomeWeights),
                                        P, P, P, ctypes.POINTER(RoutingOut), ctypes.POINTER(RoutingOut),
                                        P, S, P]
        L.uoe_layer_forward_masked.argtypes = [D, ctypes.POINTER(SmhaWeights), P, P, D, ctypes.POINTER(UomeWeights),
                                               P, P, P, P, ctypes.POINTER(RoutingOut), ctypes.POINTER(RoutingOut),
                                               P, S, P]
        for f in ("uoe_route", "uoe_route_capacity", "uoe_gather", "uoe_smha_forward", "uoe_smha_forward_masked", "uoe_uome_forward", "uoe_uome_up",
                  "uoe_uome_down", "uoe_layer_forward", "uoe_uome_backward", "uoe_smha_backward", "uoe_route_backward", "uoe_layer_backward",
                  "uoe_layer_forward_masked", "uoe_layer_backward_masked", "uoe_balance_loss", "uoe_smha_forward_steps",
                  "uoe_probe_copy", "uoe_probe_read", "uoe_probe_mfma"):
            getattr(L, f).restype = ctypes.c_int
        _lib = L
    return _lib


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def _nbytes(t) -> int:
    return int(t.numel() * t.element_size())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def _ref(d: Optional[BlockDesc]):
    return None if d is None else ctypes.byref(d)


def _done(status: int, where: str, check: bool) -> int:
    if check and status != OK:
        raise UoeError(status, where)
    return status


def block_desc(b, l, d, n, k, m, c, width, dtype, flags, rope_dim=0) -> BlockDesc:
    return BlockDesc(b, l, d, n, k, m, c, width, dtype, flags, rope_dim, (ctypes.c_int32 * 5)())


def status_string(status: int) -> str:
    return lib().uoe_status_string(int(status)).decode()


def workspace_bytes(smha: Optional[BlockDesc], uome: Optional[BlockDesc]) -> int:
    return int(lib().uoe_workspace_bytes(_ref(smha), _ref(uome)))


def route(blk, x, w_expert, w_b, w_a, noise_expert, noise_patch, expert_idx, expert_gate, patch_idx,
          patch_gate, ws, stream=None, check=True, ws_bytes=None) -> int:
    st = lib().uoe_route(_ref(blk), _ptr(x), _ptr(w_expert), _ptr(w_b), _ptr(w_a), _ptr(noise_expert),
                         _ptr(noise_patch), _ptr(expert_idx), _ptr(expert_gate), _ptr(patch_idx),
                         _ptr(patch_gate), _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes,
                         _stream(stream))
    return _done(st, "uoe_route", check)


def route_static(blk, x, w_expert, w_b, w_a, noise_expert, noise_patch, expert_idx, expert_gate, patch_idx,
                 patch_gate, stream=None, check=True) -> int:
    st = lib().uoe_route_static(_ref(blk), _ptr(x), _ptr(w_expert), _ptr(w_b), _ptr(w_a), _ptr(noise_expert),
                                _ptr(noise_patch), _ptr(expert_idx), _ptr(expert_gate), _ptr(patch_idx),
                                _ptr(patch_gate), _stream(stream))
    return _done(st, "uoe_route_static", check)


def route_capacity(blk, x, w_b, w_a, noise_patch, patch_k, capacity, load_f, load_p, ws, stream=None, check=True,
                   ws_bytes=None) -> int:
    st = lib().uoe_route_capacity(_ref(blk), _ptr(x), _ptr(w_b), _ptr(w_a), _ptr(noise_patch), int(patch_k),
                                  _ptr(capacity), _ptr(load_f), _ptr(load_p), _ptr(ws),
                                  _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    return _done(st, "uoe_route_capacity", check)


def balance_loss(blk, load_f, load_p, alpha, loss, d_patch_gate, stream=None, check=True) -> int:
    st = lib().uoe_balance_loss(_ref(blk), _ptr(load_f), _ptr(load_p), float(alpha), _ptr(loss), _ptr(d_patch_gate),
                                _stream(stream))
    return _done(st, "uoe_balance_loss", check)


def gather(blk, x, expert_idx, patch_idx, h, stream=None, check=True) -> int:
    st = lib().uoe_gather(_ref(blk), _ptr(x), _ptr(expert_idx), _ptr(patch_idx), _ptr(h), _stream(stream))
    return _done(st, "uoe_gather", check)


def smha_forward(blk, x, wq, wk, wv, wo, expert_idx, expert_gate, patch_idx, patch_gate, out, ws,
                 stream=None, check=True, ws_bytes=None) -> int:
    st = lib().uoe_smha_forward(_ref(blk), _ptr(x), _ptr(wq), _ptr(wk), _ptr(wv), _ptr(wo), _ptr(expert_idx),
                                _ptr(expert_gate), _ptr(patch_idx), _ptr(patch_gate), _ptr(out), _ptr(ws),
                                _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    return _done(st, "uoe_smha_forward", check)


def smha_forward_masked(blk, x, wq, wk, wv, wo, expert_idx, expert_gate, patch_idx, patch_gate, pad_mask, out,
                        ws, stream=None, check=True, ws_bytes=None) -> int:
    st = lib().uoe_smha_forward_masked(_ref(blk), _ptr(x), _ptr(wq), _ptr(wk), _ptr(wv), _ptr(wo),
                                       _ptr(expert_idx), _ptr(expert_gate), _ptr(patch_idx), _ptr(patch_gate),
                                       _ptr(pad_mask), _ptr(out), _ptr(ws),
                                       _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    return _done(st, "uoe_smha_forward_masked", check)


SMHA_STEP_QKV, SMHA_STEP_ATTENTION, SMHA_STEP_OUT = 1, 2, 4


def smha_forward_steps(blk, x, wq, wk, wv, wo, expert_idx, expert_gate, patch_idx, patch_gate, pad_mask, out,
                       ws, steps, stream=None, check=True, ws_bytes=None) -> int:
    st = lib().uoe_smha_forward_steps(_ref(blk), _ptr(x), _ptr(wq), _ptr(wk), _ptr(wv), _ptr(wo),
                                      _ptr(expert_idx), _ptr(expert_gate), _ptr(patch_idx), _ptr(patch_gate),
                                      _ptr(pad_mask), _ptr(out), _ptr(ws),
                                      _nbytes(ws) if ws_bytes is None else ws_bytes, int(steps), _stream(stream))
    return _done(st, "uoe_smha_forward_steps", check)


def probe_copy(src, dst, nbytes, stream=None, check=True) -> int:
    return _done(lib().uoe_probe_copy(_ptr(src), _ptr(dst), int(nbytes), _stream(stream)), "uoe_probe_copy", check)


def probe_read(src, nbytes, sink, stream=None, check=True) -> int:
    return _done(lib().uoe_probe_read(_ptr(src), int(nbytes), _ptr(sink), _stream(stream)), "uoe_probe_read", check)


def probe_mfma(operands, iters, sink, stream=None, check=True) -> float:
    """Returns the FLOP count of the launch."""
    flops = ctypes.c_double(0.0)
    _done(lib().uoe_probe_mfma(_ptr(operands), int(iters), _ptr(sink), ctypes.byref(flops), _stream(stream)),
          "uoe_probe_mfma", check)
    return float(flops.value)


def uome_forward(blk, u, a_in, a_out, expert_idx, expert_gate, patch_idx, patch_gate, out, ws,
                 stream=None, check=True, ws_bytes=None) -> int:
    st = lib().uoe_uome_forward(_ref(blk), _ptr(u), _ptr(a_in), _ptr(a_out), _ptr(expert_idx),
                                _ptr(expert_gate), _ptr(patch_idx), _ptr(patch_gate), _ptr(out), _ptr(ws),
                                _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    return _done(st, "uoe_uome_forward", check)


def uome_backward_workspace_bytes(blk) -> int:
    return int(lib().uoe_uome_backward_workspace_bytes(_ref(blk)))


def uome_backward(blk, u, a_in, a_out, expert_idx, expert_gate, patch_idx, patch_gate, d_out, d_u, d_a_in, d_a_out,
                  d_gate, d_patch_gate, ws, stream=None, check=True, ws_bytes=None) -> int:
    st = lib().uoe_uome_backward(_ref(blk), _ptr(u), _ptr(a_in), _ptr(a_out), _ptr(expert_idx), _ptr(expert_gate),
                                 _ptr(patch_idx), _ptr(patch_gate), _ptr(d_out), _ptr(d_u), _ptr(d_a_in),
                                 _ptr(d_a_out), _ptr(d_gate), _ptr(d_patch_gate), _ptr(ws),
                                 _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    return _done(st, "uoe_uome_backward", check)


def smha_backward_workspace_bytes(blk) -> int:
    return int(lib().uoe_smha_backward_workspace_bytes(_ref(blk)))


def smha_weight_grads(d_wq, d_wk, d_wv, d_wo) -> SmhaWeightGrads:
    return SmhaWeightGrads(*(_ptr(t) for t in (d_wq, d_wk, d_wv, d_wo)))


def smha_backward(blk, x, w: SmhaWeights, expert_idx, expert_gate, patch_idx, patch_gate, pad_mask, d_out, d_x,
                  dw: SmhaWeightGrads, d_expert_gate, d_patch_gate, ws, stream=None, check=True, ws_bytes=None) -> int:
    st = lib().uoe_smha_backward(_ref(blk), _ptr(x), ctypes.byref(w), _ptr(expert_idx), _ptr(expert_gate),
                                 _ptr(patch_idx), _ptr(patch_gate), _ptr(pad_mask), _ptr(d_out), _ptr(d_x), ctypes.byref(dw),
                                 _ptr(d_expert_gate), _ptr(d_patch_gate), _ptr(ws),
                                 _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    return _done(st, "uoe_smha_backward", check)


def route_backward_workspace_bytes(blk) -> int:
    return int(lib().uoe_route_backward_workspace_bytes(_ref(blk)))


def route_backward(blk, x, w_expert, w_b, w_a, expert_gate, patch_gate, d_expert_gate, d_patch_gate, d_x,
                   d_w_expert, d_w_b, d_w_a, ws, stream=None, check=True, ws_bytes=None) -> int:
    st = lib().uoe_route_backward(_ref(blk), _ptr(x), _ptr(w_expert), _ptr(w_b), _ptr(w_a), _ptr(expert_gate),
                                  _ptr(patch_gate), _ptr(d_expert_gate), _ptr(d_patch_gate), _ptr(d_x),
                                  _ptr(d_w_expert), _ptr(d_w_b), _ptr(d_w_a), _ptr(ws),
                                  _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    return _done(st, "uoe_route_backward", check)


def router_grads(d_w_expert=None, d_w_b=None, d_w_a=None) -> RouterGrads:
    return RouterGrads(*(_ptr(t) for t in (d_w_expert, d_w_b, d_w_a)))


def layer_backward_workspace_bytes(smha, uome) -> int:
    return int(lib().uoe_layer_backward_workspace_bytes(_ref(smha), _ref(uome)))


def layer_backward(smha, wa: SmhaWeights, uome, wm: UomeWeights, x, u, routing_a: RoutingOut, routing_m: RoutingOut,
                   d_out, d_x, dwa: SmhaWeightGrads, dra: Optional[RouterGrads], d_a_in, d_a_out,
                   drm: Optional[RouterGrads], ws, stream=None, check=True, ws_bytes=None) -> int:
    st = lib().uoe_layer_backward(_ref(smha), ctypes.byref(wa), _ref(uome), ctypes.byref(wm), _ptr(x), _ptr(u),
                                  ctypes.byref(routing_a), ctypes.byref(routing_m), _ptr(d_out), _ptr(d_x),
                                  ctypes.byref(dwa), None if dra is None else ctypes.byref(dra), _ptr(d_a_in),
                                  _ptr(d_a_out), None if drm is None else ctypes.byref(drm), _ptr(ws),
                                  _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    return _done(st, "uoe_layer_backward", check)


def layer_backward_masked(smha, wa: SmhaWeights, uome, wm: UomeWeights, x, pad_mask, u, routing_a: RoutingOut,
                          routing_m: RoutingOut, d_out, d_x, dwa: SmhaWeightGrads, dra: Optional[RouterGrads], d_a_in,
                          d_a_out, drm: Optional[RouterGrads], ws, stream=None, check=True, ws_bytes=None) -> int:
    st = lib().uoe_layer_backward_masked(_ref(smha), ctypes.byref(wa), _ref(uome), ctypes.byref(wm), _ptr(x),
                                         _ptr(pad_mask), _ptr(u), ctypes.byref(routing_a), ctypes.byref(routing_m),
                                         _ptr(d_out), _ptr(d_x), ctypes.byref(dwa),
                                         None if dra is None else ctypes.byref(dra), _ptr(d_a_in), _ptr(d_a_out),
                                         None if drm is None else ctypes.byref(drm), _ptr(ws),
                                         _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    return _done(st, "uoe_layer_backward_masked", check)


def uome_up(blk, u, a_in, expert_idx, expert_gate, hidden, stream=None, check=True) -> int:
    st = lib().uoe_uome_up(_ref(blk), _ptr(u), _ptr(a_in), _ptr(expert_idx), _ptr(expert_gate), _ptr(hidden),
                           _stream(stream))
    return _done(st, "uoe_uome_up", check)


def uome_down(blk, hidden, a_out, u, expert_idx, out, stream=None, check=True) -> int:
    st = lib().uoe_uome_down(_ref(blk), _ptr(hidden), _ptr(a_out), _ptr(u), _ptr(expert_idx), _ptr(out),
                             _stream(stream))
    return _done(st, "uoe_uome_down", check)


def smha_weights(w_expert, w_b, w_a, wq, wk, wv, wo) -> SmhaWeights:
    return SmhaWeights(*(_ptr(t) for t in (w_expert, w_b, w_a, wq, wk, wv, wo)))


def uome_weights(w_expert, a_in, a_out, w_b=None, w_a=None) -> UomeWeights:
    return UomeWeights(*(_ptr(t) for t in (w_expert, w_b, w_a, a_in, a_out)))


def routing_out(expert_idx=None, expert_gate=None, patch_idx=None, patch_gate=None) -> RoutingOut:
    return RoutingOut(*(_ptr(t) for t in (expert_idx, expert_gate, patch_idx, patch_gate)))


def layer_forward(smha, wa: SmhaWeights, noise_a_expert, noise_a_patch, uome, wm: UomeWeights,
                  noise_m_expert, x, out, routing_a: Optional[RoutingOut], routing_m: Optional[RoutingOut],
                  ws, stream=None, check=True, ws_bytes=None) -> int:
    st = lib().uoe_layer_forward(_ref(smha), ctypes.byref(wa) if wa is not None else None, _ptr(noise_a_expert),
                                 _ptr(noise_a_patch), _ref(uome), ctypes.byref(wm) if wm is not None else None,
                                 _ptr(noise_m_expert), _ptr(x), _ptr(out),
                                 ctypes.byref(routing_a) if routing_a is not None else None,
                                 ctypes.byref(routing_m) if routing_m is not None else None, _ptr(ws),
                                 _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    return _done(st, "uoe_layer_forward", check)


def layer_forward_masked(smha, wa: SmhaWeights, noise_a_expert, noise_a_patch, uome, wm: UomeWeights,
                         noise_m_expert, x, pad_mask, out, routing_a: Optional[RoutingOut],
                         routing_m: Optional[RoutingOut], ws, stream=None, check=True, ws_bytes=None) -> int:
    st = lib().uoe_layer_forward_masked(_ref(smha), ctypes.byref(wa) if wa is not None else None, _ptr(noise_a_expert),
                                        _ptr(noise_a_patch), _ref(uome), ctypes.byref(wm) if wm is not None else None,
                                        _ptr(noise_m_expert), _ptr(x), _ptr(pad_mask), _ptr(out),
                                        ctypes.byref(routing_a) if routing_a is not None else None,
                                        ctypes.byref(routing_m) if routing_m is not None else None, _ptr(ws),
                                        _nbytes(ws) if ws_bytes is None else ws_bytes, _stream(stream))
    return _done(st, "uoe_layer_forward_masked", check)
