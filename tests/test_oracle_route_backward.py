"""Pins for the oracle's router backward pass: central finite differences of the (already pinned)
forward routers.  L = sum(g_expert * r1) + sum(g_patch * r2) for fixed random r1, r2, so the gate
gradients handed to the routine are r1 and r2."""
import numpy as np
import pytest

import oracle


def case(seed, b=3, l=8, d=5, n=4, m=4):
    r = np.random.default_rng(seed)
    return dict(x=r.standard_normal((b, l, d)), w_e=r.standard_normal((n, l * d)) * 0.3,
                w_b=r.standard_normal((d, n)) * 0.4, w_a=r.standard_normal((l, m)) * 0.4,
                ne=r.standard_normal((b, n)), nd=r.standard_normal((b, n, m)),
                r1=r.standard_normal((b, n)), r2=r.standard_normal((b, n, m)))


def gates(cs, noise):
    _, g = oracle.expert_router(cs["x"], cs["w_e"], cs["ne"] if noise else None)
    pg = oracle.patch_gate(oracle.data_router_logits(cs["x"], cs["w_b"], cs["w_a"], cs["nd"] if noise else None))
    return g, pg


def loss(cs, noise):
    g, pg = gates(cs, noise)
    return float(np.sum(g * cs["r1"]) + np.sum(pg * cs["r2"]))


@pytest.mark.parametrize("noise", [False, True])
@pytest.mark.parametrize("seed", [0, 1])
def test_backward_matches_finite_differences(seed, noise):
    cs = case(seed)
    g, pg = gates(cs, noise)
    gr = oracle.route_backward(cs["x"], cs["w_e"], cs["w_b"], cs["w_a"], g, pg, cs["r1"], cs["r2"])
    eps = 1e-6
    rr = np.random.default_rng(50 + seed)
    for name, grad in (("x", gr.d_x), ("w_e", gr.d_w_expert), ("w_b", gr.d_w_b), ("w_a", gr.d_w_a)):
        flat = cs[name].reshape(-1)
        for idx in rr.choice(flat.size, min(flat.size, 25), replace=False):
            keep = flat[idx]
            flat[idx] = keep + eps
            lp = loss(cs, noise)
            flat[idx] = keep - eps
            lm = loss(cs, noise)
            flat[idx] = keep
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad.reshape(-1)[idx]) <= 2e-6 * max(1.0, abs(fd)), (name, idx, fd, grad.reshape(-1)[idx])


def test_each_router_alone_and_constant_shift():
    cs = case(5)
    g, pg = gates(cs, False)
    both = oracle.route_backward(cs["x"], cs["w_e"], cs["w_b"], cs["w_a"], g, pg, cs["r1"], cs["r2"])
    e_only = oracle.route_backward(cs["x"], cs["w_e"], None, None, g, None, cs["r1"], None)
    d_only = oracle.route_backward(cs["x"], None, cs["w_b"], cs["w_a"], None, pg, None, cs["r2"])
    assert np.allclose(both.d_x, e_only.d_x + d_only.d_x, rtol=0, atol=1e-12)
    assert e_only.d_w_b is None and d_only.d_w_expert is None
    # a softmax ignores a constant added to the gradient of all its outputs
    shifted = oracle.route_backward(cs["x"], cs["w_e"], cs["w_b"], cs["w_a"], g, pg, cs["r1"] + 3.0, cs["r2"] - 2.0)
    assert np.allclose(shifted.d_w_expert, both.d_w_expert, atol=1e-10) and np.allclose(shifted.d_w_a, both.d_w_a, atol=1e-10)
