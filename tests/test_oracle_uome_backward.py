"""Pins for the oracle's UoME backward pass: central finite differences of the (already pinned)
forward oracle.  L = sum(h * r) for a fixed random r, so dL/dh = r; every gradient the routine
returns is compared with (L(p + eps e) - L(p - eps e)) / (2 eps) on sampled coordinates."""
import numpy as np
import pytest

import oracle

R, GE = oracle.RESIDUAL, oracle.GATE_EXPERT


def case(seed, b=3, l=5, d=6, n=4, k=2, d_e=5):
    r = np.random.default_rng(seed)
    u = r.standard_normal((b, l, d))
    a_in = r.standard_normal((n, d, d_e)) * 0.5
    a_out = r.standard_normal((n, d_e, d)) * 0.5
    eid = np.stack([np.sort(r.choice(n, k, replace=False)) for _ in range(b)]).astype(np.int32)
    gate = r.uniform(0.2, 1.0, (b, n))
    d_out = r.standard_normal((b, l, d))
    return u, a_in, a_out, eid, gate, d_out


def loss(u, a_in, a_out, eid, gate, d_out, flags):
    return float(np.sum(oracle.uome(u, a_in, a_out, eid, gate, flags) * d_out))


@pytest.mark.parametrize("flags", [0, R, GE, R | GE])
@pytest.mark.parametrize("seed", [0, 1])
def test_backward_matches_finite_differences(flags, seed):
    u, a_in, a_out, eid, gate, d_out = case(seed)
    gr = oracle.uome_backward(u, a_in, a_out, eid, gate, d_out, flags)
    eps = 1e-6
    rr = np.random.default_rng(100 + seed)
    for name, arr, grad in (("u", u, gr.d_u), ("a_in", a_in, gr.d_a_in), ("a_out", a_out, gr.d_a_out), ("gate", gate, gr.d_gate)):
        flat = arr.reshape(-1)
        for idx in rr.choice(flat.size, min(flat.size, 25), replace=False):
            keep = flat[idx]
            flat[idx] = keep + eps
            lp = loss(u, a_in, a_out, eid, gate, d_out, flags)
            flat[idx] = keep - eps
            lm = loss(u, a_in, a_out, eid, gate, d_out, flags)
            flat[idx] = keep
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad.reshape(-1)[idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx, fd, grad.reshape(-1)[idx])


def test_unselected_experts_get_no_gradient():
    u, a_in, a_out, eid, gate, d_out = case(4, n=5, k=2)
    gr = oracle.uome_backward(u, a_in, a_out, eid, gate, d_out, R | GE)
    used = set(int(i) for row in eid for i in row)
    for i in set(range(5)) - used:
        assert not gr.d_a_in[i].any() and not gr.d_a_out[i].any()
    for bb in range(u.shape[0]):
        for i in set(range(5)) - set(int(v) for v in eid[bb]):
            assert gr.d_gate[bb, i] == 0.0
    # without the gate flag the gate has no influence
    assert not oracle.uome_backward(u, a_in, a_out, eid, gate, d_out, R).d_gate.any()


GP = oracle.GATE_PATCH


@pytest.mark.parametrize("flags", [0, R | GE, R | GP, R | GE | GP])
def test_data_selection_backward_matches_finite_differences(flags):
    """Data-selection mode: each expert sees its own patches (two experts of a sample may share one)."""
    r = np.random.default_rng(21)
    b, l, d, n, k, d_e, m, c = 2, 12, 5, 4, 2, 4, 4, 2
    u = r.standard_normal((b, l, d))
    a_in = r.standard_normal((n, d, d_e)) * 0.5
    a_out = r.standard_normal((n, d_e, d)) * 0.5
    eid = np.stack([np.sort(r.choice(n, k, replace=False)) for _ in range(b)]).astype(np.int32)
    pid = np.stack([[np.sort(r.choice(m, c, replace=False)) for _ in range(n)] for _ in range(b)]).astype(np.int32)
    pid[0, eid[0, 0]] = pid[0, eid[0, 1]]                      # a collision: both experts pick the same patches
    ge, gp = r.uniform(0.2, 1.0, (b, n)), r.uniform(0.2, 1.0, (b, n, m))
    d_out = r.standard_normal((b, l, d))
    arrs = dict(u=u, a_in=a_in, a_out=a_out, ge=ge, gp=gp)

    def loss():
        return float(np.sum(oracle.uome(u, a_in, a_out, eid, ge, flags, pid, gp, m) * d_out))

    gr = oracle.uome_backward(u, a_in, a_out, eid, ge, d_out, flags, pid, gp, m)
    eps = 1e-6
    for name, grad in (("u", gr.d_u), ("a_in", gr.d_a_in), ("a_out", gr.d_a_out), ("ge", gr.d_gate), ("gp", gr.d_patch_gate)):
        flat = arrs[name].reshape(-1)
        for idx in r.choice(flat.size, min(flat.size, 30), replace=False):
            keep = flat[idx]
            flat[idx] = keep + eps
            lp = loss()
            flat[idx] = keep - eps
            lm = loss()
            flat[idx] = keep
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad.reshape(-1)[idx]) <= 2e-6 * max(1.0, abs(fd)), (name, idx, fd, grad.reshape(-1)[idx])
