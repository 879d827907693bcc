"""Pins for the oracle's SMHA backward pass: central finite differences of the (already pinned)
forward oracle.  L = sum(u * r) for a fixed random r, so dL/du = r; every gradient the routine
returns is compared with (L(p + eps e) - L(p - eps e)) / (2 eps) on sampled coordinates, with and
without gates, the residual, the causal mask and the partial rotary embedding."""
import numpy as np
import pytest

import oracle

R, GE, GP, CA = oracle.RESIDUAL, oracle.GATE_EXPERT, oracle.GATE_PATCH, oracle.CAUSAL


def case(seed, b=2, l=12, d=6, n=3, k=2, m=4, c=2, d_h=4):
    r = np.random.default_rng(seed)
    x = r.standard_normal((b, l, d))
    w = [r.standard_normal((n, d, d_h)) * 0.6 for _ in range(3)]
    wo = r.standard_normal((n, d_h, d)) * 0.6
    eid = np.stack([np.sort(r.choice(n, k, replace=False)) for _ in range(b)]).astype(np.int32)
    pid = np.stack([[np.sort(r.choice(m, c, replace=False)) for _ in range(n)] for _ in range(b)]).astype(np.int32)
    ge = r.uniform(0.2, 1.0, (b, n))
    gp = r.uniform(0.2, 1.0, (b, n, m))
    d_out = r.standard_normal((b, l, d))
    return dict(x=x, wq=w[0], wk=w[1], wv=w[2], wo=wo, eid=eid, ge=ge, pid=pid, gp=gp, m=m, d_out=d_out)


def loss(cs, flags, rope_dim):
    u = oracle.smha(cs["x"], cs["wq"], cs["wk"], cs["wv"], cs["wo"], cs["eid"], cs["ge"], cs["pid"], cs["gp"], cs["m"],
                    flags, rope_dim)
    return float(np.sum(u * cs["d_out"]))


@pytest.mark.parametrize("flags,rope_dim", [(0, 0), (R | GE | GP, 0), (R | GE | GP | CA, 0), (GE | CA, 2), (R | GP, 4)])
@pytest.mark.parametrize("seed", [0, 1])
def test_backward_matches_finite_differences(flags, rope_dim, seed):
    cs = case(seed)
    gr = oracle.smha_backward(cs["x"], cs["wq"], cs["wk"], cs["wv"], cs["wo"], cs["eid"], cs["ge"], cs["pid"], cs["gp"],
                              cs["m"], cs["d_out"], flags, rope_dim)
    eps = 1e-6
    rr = np.random.default_rng(100 + seed)
    pairs = (("x", gr.d_x), ("wq", gr.d_wq), ("wk", gr.d_wk), ("wv", gr.d_wv), ("wo", gr.d_wo),
             ("ge", gr.d_expert_gate), ("gp", gr.d_patch_gate))
    for name, grad in pairs:
        flat = cs[name].reshape(-1)
        for idx in rr.choice(flat.size, min(flat.size, 20), replace=False):
            keep = flat[idx]
            flat[idx] = keep + eps
            lp = loss(cs, flags, rope_dim)
            flat[idx] = keep - eps
            lm = loss(cs, flags, rope_dim)
            flat[idx] = keep
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad.reshape(-1)[idx]) <= 2e-6 * max(1.0, abs(fd)), (name, idx, fd, grad.reshape(-1)[idx])


def test_collisions_and_unselected():
    """Two experts that select the same patch both send gradient to its tokens; tokens nobody
    selected get the residual's gradient only; inactive experts get none."""
    cs = case(3, n=4, k=2)
    cs["pid"][:] = np.array([0, 2], np.int32)            # every expert takes patches 0 and 2
    gr = oracle.smha_backward(cs["x"], cs["wq"], cs["wk"], cs["wv"], cs["wo"], cs["eid"], cs["ge"], cs["pid"], cs["gp"],
                              cs["m"], cs["d_out"], R | GE | GP)
    l_p = 12 // 4
    untouched = np.r_[l_p:2 * l_p, 3 * l_p:4 * l_p]
    assert np.array_equal(gr.d_x[:, untouched], cs["d_out"][:, untouched])
    assert not np.array_equal(gr.d_x[:, :l_p], cs["d_out"][:, :l_p])
    used = set(int(i) for row in cs["eid"] for i in row)
    for i in set(range(4)) - used:
        assert not gr.d_wq[i].any() and not gr.d_wo[i].any()
    assert not gr.d_patch_gate[:, :, [1, 3]].any()
    no_gate = oracle.smha_backward(cs["x"], cs["wq"], cs["wk"], cs["wv"], cs["wo"], cs["eid"], cs["ge"], cs["pid"],
                                   cs["gp"], cs["m"], cs["d_out"], R)
    assert not no_gate.d_expert_gate.any() and not no_gate.d_patch_gate.any()


@pytest.mark.parametrize("flags", [R | GE | GP, R | GE | GP | CA])
def test_backward_with_padding_mask_matches_finite_differences(flags):
    """Eq. 41: padded keys are out of every softmax; under the causal mask the first query of a unit
    whose first token is padding has no key at all and must contribute nothing."""
    cs = case(2)
    pad = np.ones((2, 12), np.uint8)
    pad[0, [0, 4, 5]] = 0
    pad[1, 9:] = 0
    gr = oracle.smha_backward(cs["x"], cs["wq"], cs["wk"], cs["wv"], cs["wo"], cs["eid"], cs["ge"], cs["pid"], cs["gp"],
                              cs["m"], cs["d_out"], flags, 0, pad)

    def loss():
        u = oracle.smha(cs["x"], cs["wq"], cs["wk"], cs["wv"], cs["wo"], cs["eid"], cs["ge"], cs["pid"], cs["gp"], cs["m"],
                        flags, 0, pad)
        return float(np.sum(u * cs["d_out"]))

    eps = 1e-6
    rr = np.random.default_rng(9)
    for name, grad in (("x", gr.d_x), ("wq", gr.d_wq), ("wk", gr.d_wk), ("wv", gr.d_wv), ("wo", gr.d_wo),
                       ("ge", gr.d_expert_gate), ("gp", gr.d_patch_gate)):
        flat = cs[name].reshape(-1)
        for idx in rr.choice(flat.size, min(flat.size, 20), replace=False):
            keep = flat[idx]
            flat[idx] = keep + eps
            lp = loss()
            flat[idx] = keep - eps
            lm = loss()
            flat[idx] = keep
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad.reshape(-1)[idx]) <= 2e-6 * max(1.0, abs(fd)), (name, idx, fd, grad.reshape(-1)[idx])
