"""Pin for the oracle's layer backward pass (the four block/router backward routines chained):
central finite differences of the whole forward oracle, out = UoME(SMHA(x)) with all four routers
live, on sampled coordinates of every parameter and of x.  A perturbation that changes a
selection (a top-k / top-c boundary crossed) is skipped: the derivative holds the selection fixed."""
import numpy as np
import pytest

import oracle
from paper_2503_02495_amd import synth

R, GE, GP, CA = oracle.RESIDUAL, oracle.GATE_EXPERT, oracle.GATE_PATCH, oracle.CAUSAL


def as_f64(inp):
    for name in ("x", "a_w_expert", "a_w_b", "a_w_a", "wq", "wk", "wv", "wo", "m_w_expert", "a_in", "a_out", "m_w_b", "m_w_a"):
        if getattr(inp, name, None) is not None:
            setattr(inp, name, np.ascontiguousarray(getattr(inp, name), np.float64))
    return inp


@pytest.mark.parametrize("fa,fm,rope_dim,noise,ds,pad", [(R | GE | GP, R | GE, 0, False, False, False),
                                                         (R | GE | GP | CA, R | GE, 2, True, False, False),
                                                         (R | GE | GP, R | GE | GP, 0, False, True, False),
                                                         (R | GE | GP | CA, R | GE, 0, False, False, True)])
def test_layer_backward_matches_finite_differences(fa, fm, rope_dim, noise, ds, pad):
    extra = dict(m_m=3, c_m=2) if ds else {}         # data-selected UoME: five routers' worth of gates live
    cfg = synth.small_config(b=2, l=12, d=8, n_a=3, d_h=4, m=4, c=2, k_a=2, n_m=3, d_e=6, k_m=2, router_noise=noise, **extra)
    inp = as_f64(synth.make_inputs(cfg, w_std=0.3))
    pm = synth.make_pad_mask(cfg, 0.25) if pad else None   # Eq. 41 inside the SMHA block of the layer
    fwd = oracle.layer_forward(inp, fa, fm, rope_dim, pm)
    r = np.random.default_rng(7).standard_normal(fwd.out.shape)
    gr = oracle.layer_backward(inp, fwd, r, fa, fm, rope_dim, pad_mask=pm)
    pairs = (("x", gr.d_x), ("wq", gr.smha.d_wq), ("wk", gr.smha.d_wk), ("wv", gr.smha.d_wv), ("wo", gr.smha.d_wo),
             ("a_w_expert", gr.route_a.d_w_expert), ("a_w_b", gr.route_a.d_w_b), ("a_w_a", gr.route_a.d_w_a),
             ("a_in", gr.uome.d_a_in), ("a_out", gr.uome.d_a_out), ("m_w_expert", gr.route_m.d_w_expert))
    if ds:
        pairs += (("m_w_b", gr.route_m.d_w_b), ("m_w_a", gr.route_m.d_w_a))
    eps, checked = 1e-6, 0
    rr = np.random.default_rng(11)

    def loss():
        f = oracle.layer_forward(inp, fa, fm, rope_dim, pm)
        same = (np.array_equal(f.routing_a.expert_id, fwd.routing_a.expert_id) and
                np.array_equal(f.routing_a.patch_id, fwd.routing_a.patch_id) and
                np.array_equal(f.routing_m.expert_id, fwd.routing_m.expert_id) and
                np.array_equal(f.routing_m.patch_id, fwd.routing_m.patch_id))
        return float(np.sum(f.out * r)), same

    for name, grad in pairs:
        flat = getattr(inp, name).reshape(-1)
        for idx in rr.choice(flat.size, min(flat.size, 12), replace=False):
            keep = flat[idx]
            flat[idx] = keep + eps
            lp, s1 = loss()
            flat[idx] = keep - eps
            lm, s2 = loss()
            flat[idx] = keep
            if not (s1 and s2):
                continue
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad.reshape(-1)[idx]) <= 5e-6 * max(1.0, abs(fd)), (name, idx, fd, grad.reshape(-1)[idx])
            checked += 1
    assert checked >= 100
