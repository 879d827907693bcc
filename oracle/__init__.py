"""CPU fp64 oracle of the Union-of-Experts layer forward pass -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``uoe_oracle.c`` (plain C, double precision, written
from the paper's Sec. III).  Only ``tests/``, the smoke check and the
``cpu_baseline`` leg of the benchmark may import this package; the GPU library
never does, and the two share no code.

Every function takes NumPy arrays, widens them to float64 and returns float64 /
int32 arrays.  The composition of a whole layer (Sec. III-C: SMHA block, then
UoME block) is written here, step by step, in the paper's order.

Parity pins: every function here is pinned by ``tests/test_oracle_*.py``
against closed forms, invariants, brute-force NumPy restatements of the
definitions and the two lossless-decomposition equivalences of Sec. III-A.  The
paper prints no worked numeric example of the layer, so absolute output values
beyond those pins are "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "uoe_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_uoe.so")

RESIDUAL = 1
GATE_EXPERT = 2
GATE_PATCH = 4
CAUSAL = 8

NEAR_TIE_REL = 1e-5  # a selection whose kept/dropped margin is below this is a near-tie


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        P = ctypes.c_void_p
        I = ctypes.c_int
        lib.uoe_oracle_set_threads.argtypes = [I]
        lib.uoe_oracle_get_threads.restype = I
        lib.uoe_oracle_data_router_logits.argtypes = [I, I, I, I, I, P, P, P, P, P]
        lib.uoe_oracle_patch_gate.argtypes = [I, I, I, P, P]
        lib.uoe_oracle_top_c.argtypes = [I, I, I, I, P, P, P]
        lib.uoe_oracle_expert_router.argtypes = [I, ctypes.c_long, I, P, P, P, P, P]
        lib.uoe_oracle_top_k.argtypes = [I, I, I, P, P, P]
        lib.uoe_oracle_expert_lists.argtypes = [I, I, I, P, P, P]
        lib.uoe_oracle_smha.argtypes = [I] * 8 + [ctypes.c_uint] + [P] * 9 + [I, P, P]
        lib.uoe_oracle_uome.argtypes = [I] * 6 + [ctypes.c_uint] + [P] * 6
        lib.uoe_oracle_uome_ds.argtypes = [I] * 8 + [ctypes.c_uint] + [P] * 8
        for f in ("data_router_logits", "patch_gate", "top_c", "expert_router", "top_k",
                  "expert_lists", "smha", "uome", "set_threads"):
            getattr(lib, "uoe_oracle_" + f).restype = None
        _lib = lib
    return _lib


def set_threads(t: int) -> None:
    _L().uoe_oracle_set_threads(int(t))


def get_threads() -> int:
    return int(_L().uoe_oracle_get_threads())


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


# --------------------------------------------------------------------------- routing
def data_router_logits(x, w_b, w_a, noise=None) -> np.ndarray:
    """Eq. 13: g'[b,i,j]; x [b,l,d], w_b [d,n], w_a [l,m]."""
    x, w_b, w_a = _f64(x), _f64(w_b), _f64(w_a)
    b, l, d = x.shape
    n, m = w_b.shape[1], w_a.shape[1]
    assert w_b.shape == (d, n) and w_a.shape == (l, m)
    nz = None if noise is None else _f64(noise)
    out = np.empty((b, n, m), np.float64)
    _L().uoe_oracle_data_router_logits(b, l, d, n, m, _p(x), _p(w_b), _p(w_a), _p(nz), _p(out))
    return out


def patch_gate(gprime) -> np.ndarray:
    """Eq. 14: softmax over the expert axis for each patch; [b,n,m] -> [b,n,m]."""
    gprime = _f64(gprime)
    b, n, m = gprime.shape
    out = np.empty_like(gprime)
    _L().uoe_oracle_patch_gate(b, n, m, _p(gprime), _p(out))
    return out


def top_c(g, c: int):
    """Eq. 17 (+ ascending sort): returns (id [b,n,c] int32, margin [b,n])."""
    g = _f64(g)
    b, n, m = g.shape
    assert 1 <= c <= m
    idx = np.empty((b, n, c), np.int32)
    margin = np.empty((b, n), np.float64)
    _L().uoe_oracle_top_c(b, n, m, c, _p(g), _p(idx), _p(margin))
    return idx, margin


def expert_router(x, w_e, noise=None):
    """Eq. 21: returns (z [b,n] logits, g [b,n] gates); x [b,l,d], w_e [n, l*d]."""
    x, w_e = _f64(x), _f64(w_e)
    b = x.shape[0]
    ld = int(np.prod(x.shape[1:]))
    n = w_e.shape[0]
    assert w_e.shape == (n, ld)
    nz = None if noise is None else _f64(noise)
    z = np.empty((b, n), np.float64)
    g = np.empty((b, n), np.float64)
    _L().uoe_oracle_expert_router(b, ld, n, _p(x), _p(w_e), _p(nz), _p(z), _p(g))
    return z, g


def top_k(g, k: int):
    """Eq. 22: returns (id [b,k] int32 ascending, margin [b])."""
    g = _f64(g)
    b, n = g.shape
    assert 1 <= k <= n
    idx = np.empty((b, k), np.int32)
    margin = np.empty((b,), np.float64)
    _L().uoe_oracle_top_k(b, n, k, _p(g), _p(idx), _p(margin))
    return idx, margin


def expert_lists(expert_id, n: int):
    """Eq. 23: per-expert sample lists; returns (counts [n], lists: list of arrays)."""
    expert_id = _i32(expert_id)
    b, k = expert_id.shape
    counts = np.empty((n,), np.int32)
    lists = np.zeros((n, b), np.int32)
    _L().uoe_oracle_expert_lists(b, n, k, _p(expert_id), _p(counts), _p(lists))
    return counts, [lists[i, :counts[i]].copy() for i in range(n)]


@dataclass
class Routing:
    expert_id: np.ndarray              # [b,k] int32 ascending
    expert_gate: np.ndarray            # [b,n]
    patch_id: np.ndarray               # [b,n,c] int32 ascending
    patch_gate: np.ndarray             # [b,n,m]
    expert_margin: np.ndarray          # [b]   (-1: nothing dropped)
    patch_margin: np.ndarray           # [b,n] (-1: nothing dropped)

    def near_ties(self, rel: float = NEAR_TIE_REL):
        """Rows whose kept/dropped margin is within `rel`: (expert rows [b], patch rows [b,n])."""
        e = (self.expert_margin >= 0) & (self.expert_margin <= rel)
        p = (self.patch_margin >= 0) & (self.patch_margin <= rel)
        return e, p


def route(x, n: int, k: int, m: int, c: int, w_expert=None, w_b=None, w_a=None,
          noise_expert=None, noise_patch=None) -> Routing:
    """Both routers of one block, reading the block input (Sec. III-B).

    k == n with no w_expert: every expert active with gate 1.  c == m with no
    w_b/w_a: every patch kept with gate 1.
    """
    x = _f64(x)
    b, l, d = x.shape
    if w_expert is None:
        assert k == n
        g_e = np.ones((b, n), np.float64)
    else:
        _, g_e = expert_router(x, w_expert, noise_expert)
    e_id, e_margin = top_k(g_e, k)
    if w_b is None:
        assert w_a is None and c == m
        g_d = np.ones((b, n, m), np.float64)
    else:
        g_d = patch_gate(data_router_logits(x, w_b, w_a, noise_patch))
    p_id, p_margin = top_c(g_d, c)
    return Routing(e_id, g_e, p_id, g_d, e_margin, p_margin)


@dataclass
class RouteGrads:
    d_x: np.ndarray            # [b,l,d]   the routers' contribution only
    d_w_expert: Optional[np.ndarray]   # [n, l*d]
    d_w_b: Optional[np.ndarray]        # [d,n]
    d_w_a: Optional[np.ndarray]        # [l,m]


def route_backward(x, w_expert, w_b, w_a, expert_gate, patch_gate_, d_expert_gate, d_patch_gate) -> RouteGrads:
    """Gradients of the two routers (Eq. 21 and Eq. 13-14) for given gradients of their gates.

    Expert router: z = W_E vec(x) (+ noise), g = softmax over the n experts; data router:
    g'[i,j] = sum_t (x W_B)[t,i] W_A[t,j] (+ noise), gate = softmax over the experts for each patch.
    The noise is additive and the top-k / top-c selections are piecewise constant, so neither
    appears here; the gates are passed in as the forward computed them.  A router that is absent
    (weights None) contributes nothing."""
    x = _f64(x)
    b, l, d = x.shape
    d_x = np.zeros_like(x)
    d_we = d_wb = d_wa = None
    if w_expert is not None:
        w_e, g, d_g = _f64(w_expert), _f64(expert_gate), _f64(d_expert_gate)
        d_z = g * (d_g - np.sum(g * d_g, axis=1, keepdims=True))        # softmax over experts
        xf = x.reshape(b, l * d)
        d_we = d_z.T @ xf
        d_x += (d_z @ w_e).reshape(b, l, d)
    if w_b is not None:
        w_b, w_a = _f64(w_b), _f64(w_a)
        pg, d_pg = _f64(patch_gate_), _f64(d_patch_gate)                # [b,n,m]
        d_l = pg * (d_pg - np.sum(pg * d_pg, axis=1, keepdims=True))    # softmax over experts, per patch
        d_wb, d_wa = np.zeros_like(w_b), np.zeros_like(w_a)
        for bb in range(b):
            t1 = x[bb] @ w_b                                            # FFN_B(x): [l,n]
            d_wa += t1 @ d_l[bb]                                        # [l,n] [n,m]
            d_t1 = w_a @ d_l[bb].T                                      # [l,m] [m,n]
            d_wb += x[bb].T @ d_t1
            d_x[bb] += d_t1 @ w_b.T
    return RouteGrads(d_x, d_we, d_wb, d_wa)


@dataclass
class Capacity:
    capacity: np.ndarray      # [b] int32, Eq. 16
    count: np.ndarray         # [b,n] int32: patches that put expert i among their top-k (Eq. 15)
    load_f: np.ndarray        # [b,n] Eq. 43
    load_p: np.ndarray        # [b,n] Eq. 44
    margin: np.ndarray        # [b,m] relative gap between the k-th and (k+1)-th logit of a patch (inf if k == n)


def capacity(gprime, k: int) -> Capacity:
    """Dynamic capacity of the two-stage routing and the balance-loss statistics.

    gprime [b,n,m]: data-router logits (Eq. 13, noise included).  Stage 1 (Eq. 15): every patch j
    picks its k experts with the highest gate g_{i,j} (Eq. 14; ties -> lower expert index).  Eq. 16:
    c = max_i #{j : i in id'_j}, per sample.  Eq. 43-44 with the patch as the routed unit:
    f_i = n/(k m) * #{j : i in id'_j}, P_i = (1/m) sum_j g_{i,j}.
    """
    gp = _f64(gprime)
    b, n, m = gp.shape
    assert 1 <= k <= n
    g = patch_gate(gp)
    cap = np.zeros(b, np.int32)
    cnt = np.zeros((b, n), np.int32)
    margin = np.full((b, m), np.inf)
    for bb in range(b):
        for j in range(m):
            col = gp[bb, :, j]                       # the gate is increasing in the logit for a fixed patch
            order = np.argsort(-col, kind="stable")  # stable: equal values keep the lower index first
            cnt[bb, order[:k]] += 1
            if k < n:
                hi, lo = col[order[k - 1]], col[order[k]]
                margin[bb, j] = (hi - lo) / max(abs(hi), abs(lo), 1e-300)
        cap[bb] = cnt[bb].max()
    return Capacity(cap, cnt, n * cnt / float(k * m), g.mean(axis=2), margin)


def balance_loss(load_f, load_p, alpha: float) -> np.ndarray:
    """Eq. 42 per sequence: L_b = alpha * sum_i f_{b,i} P_{b,i} (f, P of Eq. 43-44, [b,n] each)."""
    return float(alpha) * np.sum(_f64(load_f) * _f64(load_p), axis=1)


def balance_loss_grad(load_f, alpha: float, m: int) -> np.ndarray:
    """dL_b / d g_{b,i,j} [b,n,m] of Eq. 42: f_i (Eq. 43) is a count and passes nothing, P_i (Eq. 44)
    is the mean of the expert's m patch gates, so every patch of expert i gets alpha * f_i / m."""
    f = _f64(load_f)
    return np.repeat((float(alpha) * f / m)[:, :, None], m, axis=2)


# --------------------------------------------------------------------------- blocks
def smha(x, wq, wk, wv, wo, expert_id, expert_gate, patch_id, patch_gate_, m: int,
         flags: int = RESIDUAL, rope_dim: int = 0, pad_mask=None) -> np.ndarray:
    """Eq. 27-36 on given routing results; returns u [b,l,d].

    Optional: CAUSAL in flags (shared mask of Sec. III-C.3), rope_dim (Eq. 32, last rope_dim dims of a
    head, compacted positions), pad_mask [b,l] (1 = token, 0 = padding; Eq. 41)."""
    x, wq, wk, wv, wo = _f64(x), _f64(wq), _f64(wk), _f64(wv), _f64(wo)
    b, l, d = x.shape
    n, _, d_h = wq.shape
    expert_id, patch_id = _i32(expert_id), _i32(patch_id)
    k, c = expert_id.shape[1], patch_id.shape[2]
    assert wq.shape == wk.shape == wv.shape == (n, d, d_h) and wo.shape == (n, d_h, d)
    assert l % m == 0 and patch_id.shape == (b, n, c)
    g_e, g_d = _f64(expert_gate), _f64(patch_gate_)
    assert g_e.shape == (b, n) and g_d.shape == (b, n, m)
    assert rope_dim % 2 == 0 and 0 <= rope_dim <= d_h
    pm = None
    if pad_mask is not None:
        pm = np.ascontiguousarray(pad_mask, dtype=np.uint8)
        assert pm.shape == (b, l)
    out = np.empty((b, l, d), np.float64)
    _L().uoe_oracle_smha(b, l, d, n, k, m, c, d_h, flags, _p(x), _p(wq), _p(wk), _p(wv), _p(wo),
                         _p(expert_id), _p(g_e), _p(patch_id), _p(g_d), int(rope_dim), _p(pm), _p(out))
    return out


def uome(u, a_in, a_out, expert_id, expert_gate, flags: int = RESIDUAL, patch_id=None, patch_gate_=None,
         m: int = 1) -> np.ndarray:
    """Eq. 37-40 on given routing results; returns h [b,l,d].

    Without patch_id: expert-selection mode (every active expert sees the whole sample).  With
    patch_id [b,n,c] (and patch_gate_ [b,n,m]): each active expert sees only its c selected patches."""
    u, a_in, a_out = _f64(u), _f64(a_in), _f64(a_out)
    b, l, d = u.shape
    n, _, d_e = a_in.shape
    assert a_in.shape == (n, d, d_e) and a_out.shape == (n, d_e, d)
    expert_id = _i32(expert_id)
    k = expert_id.shape[1]
    g_e = _f64(expert_gate)
    assert g_e.shape == (b, n)
    out = np.empty((b, l, d), np.float64)
    if patch_id is None:
        assert not (flags & GATE_PATCH)
        _L().uoe_oracle_uome(b, l, d, n, k, d_e, flags, _p(u), _p(a_in), _p(a_out), _p(expert_id),
                             _p(g_e), _p(out))
        return out
    patch_id = _i32(patch_id)
    c = patch_id.shape[2]
    g_d = _f64(patch_gate_)
    assert l % m == 0 and patch_id.shape == (b, n, c) and g_d.shape == (b, n, m)
    _L().uoe_oracle_uome_ds(b, l, d, n, k, m, c, d_e, flags, _p(u), _p(a_in), _p(a_out), _p(expert_id),
                            _p(g_e), _p(patch_id), _p(g_d), _p(out))
    return out


@dataclass
class UomeGrads:
    d_u: np.ndarray        # [b,l,d]
    d_a_in: np.ndarray     # [n,d,d_e]
    d_a_out: np.ndarray    # [n,d_e,d]
    d_gate: np.ndarray     # [b,n]  (zero for experts a sample did not select, and without GATE_EXPERT)
    d_patch_gate: Optional[np.ndarray] = None   # [b,n,m] in data-selection mode (zero off the selected patches)


def uome_backward(u, a_in, a_out, expert_id, expert_gate, d_out, flags: int = RESIDUAL, patch_id=None,
                  patch_gate_=None, m: int = 1) -> UomeGrads:
    """Gradients of the UoME block (Eq. 37-40) for a given upstream gradient d_out = dL/dh [b,l,d].
    Expert-selection mode (Eq. 24-26): h[b] = (u[b]) + sum_s w * SiLU(u[b] A^I_i) A^O_i.  Data-selection
    mode (patch_id [b,n,c] given): expert i sees only the tokens T of its c selected patches and
    h[b][T_t] += w_t * (SiLU(u[b][T] A^I_i) A^O_i)_t with w_t the expert and/or patch gate of row t.

    The selections are constants of the backward pass; the gates enter as values (d_gate and
    d_patch_gate are dL/dg, to be chained into the routers by the caller)."""
    u, a_in, a_out, d_out = _f64(u), _f64(a_in), _f64(a_out), _f64(d_out)
    b, l, d = u.shape
    n, _, d_e = a_in.shape
    expert_id = _i32(expert_id)
    g = _f64(expert_gate)
    d_u = d_out.copy() if flags & RESIDUAL else np.zeros_like(u)
    d_a_in, d_a_out, d_gate = np.zeros_like(a_in), np.zeros_like(a_out), np.zeros((b, n))
    if patch_id is not None:
        patch_id, g_d = _i32(patch_id), _f64(patch_gate_)
        c, l_p = patch_id.shape[2], l // m
        d_pg = np.zeros((b, n, m))
        for bb in range(b):
            for i in expert_id[bb]:
                pid = patch_id[bb, i]
                T = (pid[:, None] * l_p + np.arange(l_p)[None, :]).reshape(-1)
                ge = g[bb, i] if flags & GATE_EXPERT else 1.0
                gp = np.repeat(g_d[bb, i, pid], l_p) if flags & GATE_PATCH else np.ones(c * l_p)
                up = u[bb, T]
                z = up @ a_in[i]
                sig = 1.0 / (1.0 + np.exp(-z))
                v = z * sig
                d_y_raw = d_out[bb, T]                       # dL/d(w_t * y_t), y = v A^O
                row_dot = np.sum((d_y_raw @ a_out[i].T) * v, axis=1)   # dL/dw_t
                if flags & GATE_EXPERT:
                    d_gate[bb, i] = np.sum(row_dot * gp)
                if flags & GATE_PATCH:
                    d_pg[bb, i, pid] = ge * row_dot.reshape(c, l_p).sum(axis=1)
                d_y = d_y_raw * (ge * gp)[:, None]
                d_a_out[i] += v.T @ d_y
                d_z = (d_y @ a_out[i].T) * (sig * (1.0 + z * (1.0 - sig)))
                d_a_in[i] += up.T @ d_z
                np.add.at(d_u[bb], T, d_z @ a_in[i].T)
        return UomeGrads(d_u, d_a_in, d_a_out, d_gate, d_pg)
    for bb in range(b):
        for i in expert_id[bb]:
            w = g[bb, i] if flags & GATE_EXPERT else 1.0
            z = u[bb] @ a_in[i]                         # [l,d_e]
            sig = 1.0 / (1.0 + np.exp(-z))
            v = z * sig                                  # SiLU(z)
            d_hp = d_out[bb]                             # dL/d(h'_i) before the weight
            d_v = w * (d_hp @ a_out[i].T)                # [l,d_e]
            if flags & GATE_EXPERT:
                d_gate[bb, i] = np.sum((v @ a_out[i]) * d_hp)
            d_a_out[i] += w * (v.T @ d_hp)
            d_z = d_v * (sig * (1.0 + z * (1.0 - sig)))  # SiLU'(z)
            d_a_in[i] += u[bb].T @ d_z
            d_u[bb] += d_z @ a_in[i].T
    return UomeGrads(d_u, d_a_in, d_a_out, d_gate)


@dataclass
class SmhaGrads:
    d_x: np.ndarray           # [b,l,d]
    d_wq: np.ndarray          # [n,d,d_h]
    d_wk: np.ndarray
    d_wv: np.ndarray
    d_wo: np.ndarray          # [n,d_h,d]
    d_expert_gate: np.ndarray  # [b,n]    zero for inactive experts and without GATE_EXPERT
    d_patch_gate: np.ndarray   # [b,n,m]  zero for patches the expert did not select and without GATE_PATCH


def _rope(a, rope_dim: int, sign: float):
    """Eq. 32 on the rows of a [rows, d_h] (row r at position r); sign = -1 applies the transposed
    (inverse) rotation, which is what the chain rule needs."""
    if rope_dim == 0:
        return a
    rows, d_h = a.shape
    first = d_h - rope_dim
    out = a.copy()
    pos = np.arange(rows, dtype=np.float64)[:, None]
    theta = 10000.0 ** (-2.0 * np.arange(rope_dim // 2, dtype=np.float64) / rope_dim)[None, :]
    cs, sn = np.cos(pos * theta), sign * np.sin(pos * theta)
    ev, od = a[:, first::2], a[:, first + 1::2]
    out[:, first::2] = ev * cs - od * sn
    out[:, first + 1::2] = ev * sn + od * cs
    return out


def smha_backward(x, wq, wk, wv, wo, expert_id, expert_gate, patch_id, patch_gate_, m: int, d_out,
                  flags: int = RESIDUAL, rope_dim: int = 0, pad_mask=None) -> SmhaGrads:
    """Gradients of the SMHA block (Eq. 27-36, with the partial RoPE of Eq. 32 and the shared causal
    mask of Sec. III-C.3) for an upstream gradient d_out = dL/du [b,l,d].

    Chain rule, per sample b and active expert i with gathered token positions T (Eq. 12, 18):
    u[T] += w_t * (softmax(q k^T / sqrt(d_h)) v) W^O_i with q, k, v = x[T] W^{q,k,v}_i (q, k rotated).
    The selections (expert_id, patch_id) are constants; the gates enter as values and their
    gradients are returned for the caller to chain into the routers.  pad_mask [b,l] (1 = token,
    0 = padding; Eq. 41) removes padded keys; a query left without any key contributes nothing."""
    x, wq, wk, wv, wo, d_out = _f64(x), _f64(wq), _f64(wk), _f64(wv), _f64(wo), _f64(d_out)
    b, l, d = x.shape
    n, _, d_h = wq.shape
    expert_id, patch_id = _i32(expert_id), _i32(patch_id)
    c = patch_id.shape[2]
    g_e, g_d = _f64(expert_gate), _f64(patch_gate_)
    l_p = l // m
    l_a = c * l_p
    scale = 1.0 / np.sqrt(float(d_h))
    gr = SmhaGrads(d_out.copy() if flags & RESIDUAL else np.zeros_like(x), np.zeros_like(wq), np.zeros_like(wk),
                   np.zeros_like(wv), np.zeros_like(wo), np.zeros((b, n)), np.zeros((b, n, m)))
    allowed = np.tril(np.ones((l_a, l_a), bool)) if flags & CAUSAL else np.ones((l_a, l_a), bool)
    for bb in range(b):
        for i in expert_id[bb]:
            pid = patch_id[bb, i]
            T = (pid[:, None] * l_p + np.arange(l_p)[None, :]).reshape(-1)
            ge = g_e[bb, i] if flags & GATE_EXPERT else 1.0
            gp = np.repeat(g_d[bb, i, pid], l_p) if flags & GATE_PATCH else np.ones(l_a)
            # forward, kept
            h = x[bb, T]
            q, kk, v = _rope(h @ wq[i], rope_dim, 1.0), _rope(h @ wk[i], rope_dim, 1.0), h @ wv[i]
            ok = allowed if pad_mask is None else allowed & (np.asarray(pad_mask)[bb, T] != 0)[None, :]
            sc = np.where(ok, (q @ kk.T) * scale, -np.inf)
            live = ok.any(axis=1, keepdims=True)
            p = np.where(ok, np.exp(sc - np.where(live, sc.max(axis=1, keepdims=True), 0.0)), 0.0)
            p /= np.where(live, p.sum(axis=1, keepdims=True), 1.0)
            o = p @ v
            y = o @ wo[i]                                   # [l_a,d] before the gates
            # backward
            d_y_raw = d_out[bb, T]                          # dL/d(w_t * y_t) = d_out at the row's token
            row_dot = np.sum(d_y_raw * y, axis=1)           # dL/dw_t
            if flags & GATE_EXPERT:
                gr.d_expert_gate[bb, i] = np.sum(row_dot * gp)
            if flags & GATE_PATCH:
                gr.d_patch_gate[bb, i, pid] = ge * row_dot.reshape(c, l_p).sum(axis=1)
            d_y = d_y_raw * (ge * gp)[:, None]
            gr.d_wo[i] += o.T @ d_y
            d_o = d_y @ wo[i].T
            gr_v = p.T @ d_o
            d_p = d_o @ v.T
            d_s = p * (d_p - np.sum(d_p * p, axis=1, keepdims=True))   # softmax backward, masked entries have p = 0
            d_q = _rope((d_s @ kk) * scale, rope_dim, -1.0)
            d_k = _rope((d_s.T @ q) * scale, rope_dim, -1.0)
            gr.d_wq[i] += h.T @ d_q
            gr.d_wk[i] += h.T @ d_k
            gr.d_wv[i] += h.T @ gr_v
            np.add.at(gr.d_x[bb], T, d_q @ wq[i].T + d_k @ wk[i].T + gr_v @ wv[i].T)
    return gr


@dataclass
class LayerResult:
    routing_a: Routing
    u: np.ndarray
    routing_m: Routing
    out: np.ndarray


def layer_forward(inp, flags_a: int = RESIDUAL | GATE_EXPERT | GATE_PATCH,
                  flags_m: int = RESIDUAL | GATE_EXPERT, rope_dim: int = 0, pad_mask=None) -> LayerResult:
    """One UoE layer (Sec. III-C): out = UoME(SMHA(x)); `inp` is a LayerInputs-like object.

    The UoME router reads u, the finished SMHA output.  pad_mask [b,l] (Eq. 41) acts inside the
    attention of the SMHA block only.
    """
    cfg = inp.cfg
    ra = route(inp.x, cfg.n_a, cfg.k_a, cfg.m, cfg.c, inp.a_w_expert, inp.a_w_b, inp.a_w_a,
               inp.noise_a_expert, inp.noise_a_patch)
    u = smha(inp.x, inp.wq, inp.wk, inp.wv, inp.wo, ra.expert_id, ra.expert_gate, ra.patch_id,
             ra.patch_gate, cfg.m, flags_a, rope_dim, pad_mask)
    if getattr(cfg, "m_m", 1) > 1:  # UoME with patch-wise data selection (Eq. 37)
        rm = route(u, cfg.n_m, cfg.k_m, cfg.m_m, cfg.c_m, inp.m_w_expert, inp.m_w_b, inp.m_w_a,
                   inp.noise_m_expert, inp.noise_m_patch)
        out = uome(u, inp.a_in, inp.a_out, rm.expert_id, rm.expert_gate, flags_m, rm.patch_id, rm.patch_gate, cfg.m_m)
    else:
        rm = route(u, cfg.n_m, cfg.k_m, 1, 1, inp.m_w_expert, None, None, inp.noise_m_expert, None)
        out = uome(u, inp.a_in, inp.a_out, rm.expert_id, rm.expert_gate, flags_m)
    return LayerResult(ra, u, rm, out)


@dataclass
class LayerGrads:
    d_x: np.ndarray
    smha: SmhaGrads            # block weights (d_x, gate members: the block's own share)
    route_a: RouteGrads        # SMHA routers
    uome: UomeGrads            # d_u member: dL/du before the UoME router's share is added
    route_m: RouteGrads        # UoME router


def layer_backward(inp, fwd: LayerResult, d_out, flags_a: int = RESIDUAL | GATE_EXPERT | GATE_PATCH,
                   flags_m: int = RESIDUAL | GATE_EXPERT, rope_dim: int = 0, gates_a=None, gate_m=None,
                   patch_gate_m=None, pad_mask=None) -> LayerGrads:
    """Gradients of layer_forward for d_out = dL/d(out): the chain rule through
    out = UoME(u; routers on u), u = SMHA(x; routers on x), the selections held constant.

    `fwd` is the forward result whose routing is differentiated through; gates_a = (expert, patch)
    and gate_m override the gate VALUES used (a test passes the fp32-rounded gates the device gets);
    pad_mask is the forward call's (Eq. 41)."""
    cfg = inp.cfg
    ra, rm = fwd.routing_a, fwd.routing_m
    ge_a, gp_a = (ra.expert_gate, ra.patch_gate) if gates_a is None else gates_a
    ge_m = rm.expert_gate if gate_m is None else gate_m
    if getattr(cfg, "m_m", 1) > 1:   # UoME with patch-wise data selection: its data router is live too
        gp_m = rm.patch_gate if patch_gate_m is None else patch_gate_m
        gm = uome_backward(fwd.u, inp.a_in, inp.a_out, rm.expert_id, ge_m, d_out, flags_m, rm.patch_id, gp_m, cfg.m_m)
        rgm = route_backward(fwd.u, inp.m_w_expert, inp.m_w_b, inp.m_w_a, ge_m, gp_m, gm.d_gate, gm.d_patch_gate)
    else:
        gm = uome_backward(fwd.u, inp.a_in, inp.a_out, rm.expert_id, ge_m, d_out, flags_m)
        if inp.m_w_expert is not None:
            rgm = route_backward(fwd.u, inp.m_w_expert, None, None, ge_m, None, gm.d_gate, None)
        else:
            rgm = RouteGrads(np.zeros_like(gm.d_u), None, None, None)
    d_u = gm.d_u + rgm.d_x
    ga = smha_backward(inp.x, inp.wq, inp.wk, inp.wv, inp.wo, ra.expert_id, ge_a, ra.patch_id, gp_a, cfg.m, d_u,
                       flags_a, rope_dim, pad_mask)
    rga = route_backward(inp.x, inp.a_w_expert, inp.a_w_b, inp.a_w_a, ge_a, gp_a, ga.d_expert_gate, ga.d_patch_gate)
    return LayerGrads(ga.d_x + rga.d_x, ga, rga, gm, rgm)
