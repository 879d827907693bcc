"""Pins for the oracle's UoME with patch-wise data selection (Eq. 37-40 in full).

The MLP acts on every token independently, so the data-selected block has a plain per-token
definition: out[b,t] = u[b,t] + sum over active experts i that selected the patch of t of
w(b,i,patch) * SiLU(u[b,t] A^I_i) A^O_i.  That definition is written out here with NumPy
(no gather, no scatter) and does not call or copy the oracle; further pins: all patches selected
reduces to the undecomposed dense MLP and to the expert-selection routine, the order in which the
routing lists a patch does not matter, gate weights enter linearly.
"""
import numpy as np
import pytest

import oracle
from paper_2503_02495_amd import synth

R, GE, GP = oracle.RESIDUAL, oracle.GATE_EXPERT, oracle.GATE_PATCH


def silu(z):
    return z / (1.0 + np.exp(-z))


def per_token_definition(u, a_in, a_out, eid, ge, pid, gd, m, flags):
    b, l, d = u.shape
    n = a_in.shape[0]
    l_p = l // m
    out = u.copy() if flags & R else np.zeros_like(u)
    for bb in range(b):
        for t in range(l):
            p = t // l_p
            for i in eid[bb]:
                if p not in pid[bb, i]:
                    continue
                w = (ge[bb, i] if flags & GE else 1.0) * (gd[bb, i, p] if flags & GP else 1.0)
                out[bb, t] += w * (silu(u[bb, t] @ a_in[i]) @ a_out[i])
    return out


def random_case(seed, b=3, l=24, d=10, n=5, k=3, m=6, c=2, d_e=7):
    r = np.random.default_rng(seed)
    u = r.standard_normal((b, l, d))
    a_in = r.standard_normal((n, d, d_e)) * 0.4
    a_out = r.standard_normal((n, d_e, d)) * 0.4
    eid = np.stack([np.sort(r.choice(n, k, replace=False)) for _ in range(b)]).astype(np.int32)
    pid = np.stack([[np.sort(r.choice(m, c, replace=False)) for _ in range(n)] for _ in range(b)]).astype(np.int32)
    ge = r.uniform(0.1, 1.0, (b, n))
    gd = r.uniform(0.1, 1.0, (b, n, m))
    return u, a_in, a_out, eid, ge, pid, gd


@pytest.mark.parametrize("flags", [0, R, R | GE, R | GP, R | GE | GP, GE | GP])
@pytest.mark.parametrize("seed", [0, 1])
def test_matches_the_per_token_definition(flags, seed):
    u, a_in, a_out, eid, ge, pid, gd = random_case(seed)
    got = oracle.uome(u, a_in, a_out, eid, ge, flags, pid, gd, m=6)
    want = per_token_definition(u, a_in, a_out, eid, ge, pid, gd, 6, flags)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_ragged_shapes_and_single_patch_rows():
    # l_p = 1 (every token its own patch), c = 1, k = n
    u, a_in, a_out, eid, ge, pid, gd = random_case(5, b=2, l=7, d=4, n=3, k=3, m=7, c=1, d_e=5)
    got = oracle.uome(u, a_in, a_out, eid, ge, R | GE | GP, pid, gd, m=7)
    want = per_token_definition(u, a_in, a_out, eid, ge, pid, gd, 7, R | GE | GP)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_all_patches_selected_is_the_dense_mlp_and_the_expert_selection_block():
    r = np.random.default_rng(3)
    b, l, d, n, m, d_e = 2, 12, 6, 4, 3, 5
    u = r.standard_normal((b, l, d))
    a_in, a_out = r.standard_normal((n, d, d_e)) * 0.5, r.standard_normal((n, d_e, d)) * 0.5
    eid = np.tile(np.arange(n, dtype=np.int32), (b, 1))
    pid = np.tile(np.arange(m, dtype=np.int32), (b, n, 1))
    ge, gd = np.ones((b, n)), np.ones((b, n, m))
    got = oracle.uome(u, a_in, a_out, eid, ge, R, pid, gd, m=m)
    z = u @ np.concatenate(list(a_in), axis=1)                      # undecomposed two-layer MLP
    dense = u + silu(z) @ np.concatenate(list(a_out), axis=0)
    np.testing.assert_allclose(got, dense, rtol=1e-12, atol=1e-12)
    # with k < n and expert gates it is the expert-selection routine on the same routing
    eid2 = np.array([[0, 2], [1, 3]], np.int32)
    ge2 = r.uniform(0.2, 1.0, (b, n))
    np.testing.assert_allclose(oracle.uome(u, a_in, a_out, eid2, ge2, R | GE, pid, gd, m=m),
                               oracle.uome(u, a_in, a_out, eid2, ge2, R | GE), rtol=1e-12, atol=1e-12)


def test_listing_order_of_patches_does_not_matter_and_gates_are_linear():
    u, a_in, a_out, eid, ge, pid, gd = random_case(7)
    base = oracle.uome(u, a_in, a_out, eid, ge, GE | GP, pid, gd, m=6)
    np.testing.assert_allclose(oracle.uome(u, a_in, a_out, eid, ge, GE | GP, pid[:, :, ::-1].copy(), gd, m=6), base,
                               rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.uome(u, a_in, a_out, eid, ge, GE | GP, pid, 3.0 * gd, m=6), 3.0 * base,
                               rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.uome(u, a_in, a_out, eid, 0.5 * ge, GE | GP, pid, gd, m=6), 0.5 * base,
                               rtol=1e-12, atol=1e-12)
    # tokens of patches nobody selected only carry the residual
    out = oracle.uome(u, a_in, a_out, eid, ge, R | GE | GP, pid, gd, m=6)
    l_p = u.shape[1] // 6
    for bb in range(u.shape[0]):
        chosen = set(int(p) for i in eid[bb] for p in pid[bb, i])
        for p in set(range(6)) - chosen:
            np.testing.assert_array_equal(out[bb, p * l_p:(p + 1) * l_p], u[bb, p * l_p:(p + 1) * l_p])


def test_layer_composition_with_data_selected_uome():
    cfg = synth.small_config(b=2, l=24, d=16, n_a=3, d_h=8, m=4, c=2, k_a=2, n_m=4, d_e=8, k_m=2, m_m=6, c_m=3)
    inp = synth.make_inputs(cfg, w_std=0.3)
    res = oracle.layer_forward(inp)
    rm = oracle.route(res.u, cfg.n_m, cfg.k_m, cfg.m_m, cfg.c_m, inp.m_w_expert, inp.m_w_b, inp.m_w_a, None, None)
    np.testing.assert_array_equal(rm.patch_id, res.routing_m.patch_id)
    want = per_token_definition(res.u, inp.a_in.astype(np.float64), inp.a_out.astype(np.float64), rm.expert_id,
                                rm.expert_gate, rm.patch_id, rm.patch_gate, cfg.m_m, R | GE)
    np.testing.assert_allclose(res.out, want, rtol=1e-11, atol=1e-11)


def test_inputs_of_existing_configs_are_unchanged_by_the_new_fields():
    # the data-selection tensors are drawn last, so (config, seed) still names the same base tensors
    a = synth.make_inputs(synth.small_config(seed=9))
    bcfg = synth.small_config(seed=9, m_m=4, c_m=2)
    b = synth.make_inputs(bcfg)
    for f in ("x", "a_w_expert", "a_w_b", "a_w_a", "wq", "wo", "m_w_expert", "a_in", "a_out"):
        np.testing.assert_array_equal(getattr(a, f), getattr(b, f))
    assert a.m_w_b is None and b.m_w_b.shape == (bcfg.d, bcfg.n_m) and b.m_w_a.shape == (bcfg.l, 4)
