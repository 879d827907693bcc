"""Seeded synthetic inputs for one Union-of-Experts layer.

This module only *draws numbers and shapes them*: it contains none of the
method's arithmetic (no router, no softmax, no selection, no matmul), so both
the CPU oracle's tests and the HIP path's tests can take their inputs from it
without sharing any computation.

Notation follows the paper (Sec. III-B/III-C): b batch, l sequence length,
d model dim; SMHA block: n_a head-experts of dim d_h, m patches of l_p = l/m
tokens, c patches kept per expert, k_a experts kept per sample; UoME block:
n_m MLP experts of hidden dim d_e, k_m kept per sample.

Draw order is fixed (x; SMHA W_E, W_B, W_A, W^q, W^k, W^v, W^o; UoME W_E, A^I,
A^O; then the optional router-noise tensors; then, for configs with UoME data
selection, its W_B, W_A and patch noise) so a (config, seed) pair names one
input set.  x ~ N(0,1); every weight ~ N(0, std 0.02).  For bf16 configs each
tensor is rounded once to bfloat16 (round to nearest, ties to even) here on
the host; both sides consume exactly those rounded values.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

F32 = "f32"
BF16 = "bf16"


@dataclass(frozen=True)
class LayerConfig:
    name: str
    b: int
    l: int
    d: int
    # SMHA block
    n_a: int
    d_h: int
    m: int
    c: int
    k_a: int
    # UoME block
    n_m: int
    d_e: int
    k_m: int
    dtype: str = BF16
    seed: int = 0
    router_noise: bool = False
    # UoME patch-wise data selection (Eq. 37): m_m patches, c_m kept per expert; 1/1 = expert selection only
    m_m: int = 1
    c_m: int = 1

    @property
    def l_p(self) -> int:
        return self.l // self.m

    @property
    def l_a(self) -> int:
        return self.c * self.l_p

    @property
    def tokens(self) -> int:
        return self.b * self.l


# The five workload shapes: a tiny fp32 case the oracle finishes at once, a
# language-modeling shape, a long-range shape, a ViT-style image shape (14x14
# patch tokens, one image row per routing patch) and a large shape.
CONFIGS: Dict[str, LayerConfig] = {
    "tiny": LayerConfig("tiny", b=2, l=64, d=64, n_a=4, d_h=16, m=8, c=2, k_a=2,
                        n_m=4, d_e=64, k_m=2, dtype=F32, seed=0),
    "lm": LayerConfig("lm", b=8, l=512, d=512, n_a=8, d_h=64, m=16, c=4, k_a=4,
                      n_m=8, d_e=256, k_m=4, dtype=BF16, seed=1),
    "longrange": LayerConfig("longrange", b=16, l=4096, d=256, n_a=8, d_h=32, m=64, c=8, k_a=2,
                             n_m=8, d_e=128, k_m=2, dtype=BF16, seed=2),
    "vit": LayerConfig("vit", b=128, l=196, d=384, n_a=6, d_h=64, m=14, c=4, k_a=3,
                       n_m=6, d_e=256, k_m=3, dtype=BF16, seed=3),
    "large": LayerConfig("large", b=4, l=8192, d=1024, n_a=16, d_h=64, m=128, c=16, k_a=8,
                         n_m=16, d_e=256, k_m=8, dtype=BF16, seed=4, router_noise=True),
}
CONFIG_ORDER = ["tiny", "lm", "longrange", "vit", "large"]


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 -> nearest bfloat16 (ties to even), returned as float32 values.

    Inputs are finite by contract, so no NaN handling is needed.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Bit patterns (uint16) of float32 values that are already bf16-exact."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    assert not np.any(bits & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (bits >> np.uint32(16)).astype(np.uint16)


@dataclass
class LayerInputs:
    cfg: LayerConfig
    x: np.ndarray                      # [b, l, d]
    # SMHA
    a_w_expert: np.ndarray             # [n_a, l*d]   expert-selection router
    a_w_b: np.ndarray                  # [d, n_a]     data-selection router, first map
    a_w_a: np.ndarray                  # [l, m]       data-selection router, second map
    wq: np.ndarray                     # [n_a, d, d_h]
    wk: np.ndarray
    wv: np.ndarray
    wo: np.ndarray                     # [n_a, d_h, d]
    # UoME
    m_w_expert: np.ndarray             # [n_m, l*d]
    a_in: np.ndarray                   # [n_m, d, d_e]
    a_out: np.ndarray                  # [n_m, d_e, d]
    # optional additive router-logit noise (fp32, never rounded to bf16)
    noise_a_expert: Optional[np.ndarray] = None    # [b, n_a]
    noise_a_patch: Optional[np.ndarray] = None     # [b, n_a, m]
    noise_m_expert: Optional[np.ndarray] = None    # [b, n_m]
    # UoME data-selection router (only when cfg.m_m > 1)
    m_w_b: Optional[np.ndarray] = None             # [d, n_m]
    m_w_a: Optional[np.ndarray] = None             # [l, m_m]
    noise_m_patch: Optional[np.ndarray] = None     # [b, n_m, m_m]
    extras: dict = field(default_factory=dict)


def _draw(rng: np.random.Generator, shape, std: float, dtype: str) -> np.ndarray:
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if dtype == BF16:
        a = round_to_bf16(a)
    return a


def make_inputs(cfg: LayerConfig, seed: Optional[int] = None, w_std: float = 0.02) -> LayerInputs:
    """All tensors of one layer call, as float32 arrays (bf16-exact for bf16 configs)."""
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    dt = cfg.dtype
    b, l, d = cfg.b, cfg.l, cfg.d
    x = _draw(rng, (b, l, d), 1.0, dt)
    a_w_expert = _draw(rng, (cfg.n_a, l * d), w_std, dt)
    a_w_b = _draw(rng, (d, cfg.n_a), w_std, dt)
    a_w_a = _draw(rng, (l, cfg.m), w_std, dt)
    wq = _draw(rng, (cfg.n_a, d, cfg.d_h), w_std, dt)
    wk = _draw(rng, (cfg.n_a, d, cfg.d_h), w_std, dt)
    wv = _draw(rng, (cfg.n_a, d, cfg.d_h), w_std, dt)
    wo = _draw(rng, (cfg.n_a, cfg.d_h, d), w_std, dt)
    m_w_expert = _draw(rng, (cfg.n_m, l * d), w_std, dt)
    a_in = _draw(rng, (cfg.n_m, d, cfg.d_e), w_std, dt)
    a_out = _draw(rng, (cfg.n_m, cfg.d_e, d), w_std, dt)
    inp = LayerInputs(cfg, x, a_w_expert, a_w_b, a_w_a, wq, wk, wv, wo, m_w_expert, a_in, a_out)
    if cfg.router_noise:
        inp.noise_a_expert = rng.standard_normal(size=(b, cfg.n_a), dtype=np.float32)
        inp.noise_a_patch = rng.standard_normal(size=(b, cfg.n_a, cfg.m), dtype=np.float32)
        inp.noise_m_expert = rng.standard_normal(size=(b, cfg.n_m), dtype=np.float32)
    if cfg.m_m > 1:
        inp.m_w_b = _draw(rng, (d, cfg.n_m), w_std, dt)
        inp.m_w_a = _draw(rng, (l, cfg.m_m), w_std, dt)
        if cfg.router_noise:
            inp.noise_m_patch = rng.standard_normal(size=(b, cfg.n_m, cfg.m_m), dtype=np.float32)
    return inp


def make_upstream_grad(cfg: LayerConfig, seed: Optional[int] = None) -> np.ndarray:
    """A synthetic upstream gradient dL/d(out) [b,l,d] for backward-pass tests and timing: unit
    normal, bf16-exact for bf16 configs, from a stream separate from make_inputs'."""
    rng = np.random.default_rng((cfg.seed if seed is None else seed) + 7919)
    return _draw(rng, (cfg.b, cfg.l, cfg.d), 1.0, cfg.dtype)


def make_gate_grads(cfg: LayerConfig, n: int, m: int, seed: Optional[int] = None):
    """Synthetic gradients of a block's gates, (d_expert_gate [b,n], d_patch_gate [b,n,m]) float32,
    for the router backward tests: unit normal, from a stream of their own."""
    rng = np.random.default_rng((cfg.seed if seed is None else seed) + 104729)
    return (rng.standard_normal(size=(cfg.b, n), dtype=np.float32),
            rng.standard_normal(size=(cfg.b, n, m), dtype=np.float32))


def make_pad_mask(cfg: LayerConfig, pad_frac: float, seed: Optional[int] = None) -> np.ndarray:
    """A synthetic padding mask [b,l] uint8 (1 = token, 0 = padding): tokens padded at random with
    probability pad_frac, plus a padded run over the first half of sample 0 (whole units lose all
    their early keys)."""
    rng = np.random.default_rng((cfg.seed if seed is None else seed) + 15485863)
    pad = (rng.random((cfg.b, cfg.l)) >= pad_frac).astype(np.uint8)
    pad[0, : cfg.l // 2] = 0
    return pad


def small_config(name: str = "small", **kw) -> LayerConfig:
    """A config with every size overridable, for randomly drawn tiny shapes in tests."""
    base = dict(b=2, l=24, d=16, n_a=3, d_h=8, m=4, c=2, k_a=2, n_m=3, d_e=8, k_m=2,
                dtype=F32, seed=0, router_noise=False, m_m=1, c_m=1)
    base.update(kw)
    return LayerConfig(name, **base)
