"""Pins for the oracle's routing functions (Sec. III-B: Eq. 13-17, 21-23).

Each pin is something other than the oracle itself: a closed form, an
invariant, a crafted case with a known answer, or a brute-force NumPy
restatement of the definition (einsum / full stable sort) on tiny inputs.
"""
import numpy as np
import pytest

import oracle
from paper_2503_02495_amd import synth


def rng(seed=0):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------- Eq. 13
def test_data_router_matches_einsum_definition():
    r = rng(1)
    b, l, d, n, m = 3, 28, 10, 5, 7
    x = r.standard_normal((b, l, d))
    w_b = r.standard_normal((d, n))
    w_a = r.standard_normal((l, m))
    want = np.einsum("bte,ei,tj->bij", x, w_b, w_a)
    got = oracle.data_router_logits(x, w_b, w_a)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    noise = r.standard_normal((b, n, m))
    np.testing.assert_allclose(oracle.data_router_logits(x, w_b, w_a, noise), want + noise,
                               rtol=1e-12, atol=1e-12)


def test_data_router_mean_pool_closed_form():
    """W_A = block mean-pool  =>  g'[b,i,j] = mean over patch j of (x W_B)[.,i]."""
    r = rng(2)
    b, m, l_p, d, n = 2, 4, 6, 5, 3
    l = m * l_p
    x = r.standard_normal((b, l, d))
    w_b = r.standard_normal((d, n))
    w_a = np.zeros((l, m))
    for j in range(m):
        w_a[j * l_p:(j + 1) * l_p, j] = 1.0 / l_p
    got = oracle.data_router_logits(x, w_b, w_a)
    want = np.empty((b, n, m))
    for bb in range(b):
        proj = x[bb] @ w_b                          # [l, n]
        for j in range(m):
            want[bb, :, j] = proj[j * l_p:(j + 1) * l_p].mean(axis=0)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_data_router_not_transposed():
    """A one-hot W_B / W_A picks out exactly x[b, t0, e0] at [i0, j0] (catches swapped axes)."""
    b, l, d, n, m = 2, 6, 4, 3, 2
    x = rng(3).standard_normal((b, l, d))
    w_b = np.zeros((d, n)); w_b[2, 1] = 1.0
    w_a = np.zeros((l, m)); w_a[4, 0] = 1.0
    got = oracle.data_router_logits(x, w_b, w_a)
    want = np.zeros((b, n, m)); want[:, 1, 0] = x[:, 4, 2]
    np.testing.assert_allclose(got, want, atol=0)


# ----------------------------------------------------------------- Eq. 14
def test_patch_gate_is_softmax_over_experts():
    g = rng(4).standard_normal((3, 5, 7)) * 3
    p = oracle.patch_gate(g)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=1e-14)          # sums over EXPERTS
    assert not np.allclose(p.sum(axis=2), 1.0)                           # not over patches
    np.testing.assert_allclose(oracle.patch_gate(g + 100.0), p, rtol=1e-12)   # shift invariance
    e = np.exp(g)
    np.testing.assert_allclose(p, e / e.sum(axis=1, keepdims=True), rtol=1e-13)
    # two experts: closed form is the logistic of the logit difference
    g2 = rng(5).standard_normal((2, 2, 3))
    p2 = oracle.patch_gate(g2)
    np.testing.assert_allclose(p2[:, 0], 1.0 / (1.0 + np.exp(g2[:, 1] - g2[:, 0])), rtol=1e-13)


# ----------------------------------------------------------------- Eq. 21
def test_expert_router_one_hot_and_linearity():
    r = rng(6)
    b, l, d, n = 3, 5, 4, 4
    x = r.standard_normal((b, l, d))
    w = np.zeros((n, l * d))
    picks = [(0, 0), (2, 3), (4, 1), (1, 2)]
    for i, (t, e) in enumerate(picks):
        w[i, t * d + e] = 1.0                      # row-major flattening of [l, d]
    z, g = oracle.expert_router(x, w)
    for i, (t, e) in enumerate(picks):
        np.testing.assert_allclose(z[:, i], x[:, t, e], atol=0)
    np.testing.assert_allclose(g.sum(axis=1), 1.0, rtol=1e-14)
    w = r.standard_normal((n, l * d))
    z1, _ = oracle.expert_router(x, w)
    np.testing.assert_allclose(z1, x.reshape(b, -1) @ w.T, rtol=1e-12, atol=1e-12)
    x2 = r.standard_normal((b, l, d))
    z2, _ = oracle.expert_router(x2, w)
    z12, g12 = oracle.expert_router(2.0 * x - 3.0 * x2, w)
    np.testing.assert_allclose(z12, 2.0 * z1 - 3.0 * z2, rtol=1e-11, atol=1e-11)
    e = np.exp(z12 - z12.max(axis=1, keepdims=True))
    np.testing.assert_allclose(g12, e / e.sum(axis=1, keepdims=True), rtol=1e-13)
    noise = r.standard_normal((b, n))
    zn, _ = oracle.expert_router(x, w, noise)
    np.testing.assert_allclose(zn, z1 + noise, rtol=1e-12, atol=1e-12)


# ----------------------------------------------------------------- Eq. 17 / 22
def brute_top(values, keep):
    """Full stable sort by (-value, index); keep the first `keep`; report ascending."""
    order = sorted(range(len(values)), key=lambda j: (-values[j], j))
    return sorted(order[:keep])


def check_selection_invariants(v, idx, keep):
    idx = list(idx)
    assert len(idx) == keep and len(set(idx)) == keep
    assert idx == sorted(idx) and 0 <= idx[0] and idx[-1] < len(v)
    kept = set(idx)
    dropped = [j for j in range(len(v)) if j not in kept]
    for j in dropped:
        assert all(v[i] >= v[j] for i in idx)                 # every kept >= every dropped
        for i in idx:
            if v[i] == v[j]:
                assert i < j                                   # equal values: lower index kept


def test_top_c_crafted_cases():
    m = 8
    flat = np.ones((1, 1, m))
    idx, margin = oracle.top_c(flat, 3)
    assert idx.tolist() == [[[0, 1, 2]]] and margin[0, 0] == 0.0       # all equal -> 0..c-1
    inc = np.arange(m, dtype=float).reshape(1, 1, m)
    assert oracle.top_c(inc, 3)[0].tolist() == [[[5, 6, 7]]]           # increasing -> last c
    dec = inc[:, :, ::-1].copy()
    assert oracle.top_c(dec, 3)[0].tolist() == [[[0, 1, 2]]]
    # duplicates straddling the cut: values 5 at 1,4,6 ; keep 2 of the three after the 9
    v = np.array([[[1.0, 5.0, 9.0, 0.0, 5.0, 2.0, 5.0, 3.0]]])
    assert oracle.top_c(v, 3)[0].tolist() == [[[1, 2, 4]]]
    # keep everything
    idx, margin = oracle.top_c(v, m)
    assert idx.tolist() == [[list(range(m))]] and margin[0, 0] == -1.0


def test_top_c_and_top_k_match_brute_force():
    r = rng(7)
    for trial in range(40):
        b, n, m = r.integers(1, 4), r.integers(1, 7), r.integers(1, 15)
        c = int(r.integers(1, m + 1))
        g = r.standard_normal((b, n, m))
        if trial % 3 == 0:                         # many exact ties
            g = np.round(g * 2) / 2
        idx, _ = oracle.top_c(g, c)
        for bb in range(b):
            for i in range(n):
                assert idx[bb, i].tolist() == brute_top(g[bb, i], c)
                check_selection_invariants(g[bb, i], idx[bb, i], c)
        k = int(r.integers(1, n + 1))
        ge = g[:, :, 0].copy()
        kid, _ = oracle.top_k(ge, k)
        for bb in range(b):
            assert kid[bb].tolist() == brute_top(ge[bb], k)
            check_selection_invariants(ge[bb], kid[bb], k)


def test_top_c_uses_gate_values_not_logits():
    """The normaliser differs per patch, so ranking patches by gate differs from ranking by logit."""
    gprime = np.array([[[2.0, 1.0],          # expert 0: larger logit on patch 0 ...
                        [5.0, -3.0]]])       # ... but expert 1 dominates patch 0's softmax
    g = oracle.patch_gate(gprime)
    assert gprime[0, 0, 0] > gprime[0, 0, 1] and g[0, 0, 0] < g[0, 0, 1]
    assert oracle.top_c(g, 1)[0][0, 0].tolist() == [1]


def test_near_tie_margin_and_flag():
    base = np.array([[[0.5, 0.25, 0.125, 0.125]]])
    for rel, flagged in ((0.5e-5, True), (2e-5, False)):
        v = base.copy()
        v[0, 0, 2] = 0.25 * (1.0 - rel)            # first dropped value when c = 2
        idx, margin = oracle.top_c(v, 2)
        assert idx[0, 0].tolist() == [0, 1]
        np.testing.assert_allclose(margin[0, 0], rel, rtol=1e-9)
        rt = oracle.Routing(np.zeros((1, 1), np.int32), np.ones((1, 1)), idx, v,
                            np.array([-1.0]), margin)
        assert bool(rt.near_ties()[1][0, 0]) is flagged and not rt.near_ties()[0][0]


def test_expert_lists():
    eid = np.array([[0, 2], [1, 2], [0, 1], [2, 3]], np.int32)
    counts, lists = oracle.expert_lists(eid, 4)
    assert counts.tolist() == [2, 2, 3, 1]
    assert [l.tolist() for l in lists] == [[0, 2], [1, 2], [0, 1, 3], [3]]
    assert counts.sum() == eid.size


# ----------------------------------------------------------------- composed routing
@pytest.mark.parametrize("name", ["tiny"])
def test_route_invariants_on_config(name):
    cfg = synth.CONFIGS[name]
    inp = synth.make_inputs(cfg)
    rt = oracle.route(inp.x, cfg.n_a, cfg.k_a, cfg.m, cfg.c, inp.a_w_expert, inp.a_w_b, inp.a_w_a)
    assert rt.expert_id.shape == (cfg.b, cfg.k_a) and rt.patch_id.shape == (cfg.b, cfg.n_a, cfg.c)
    for bb in range(cfg.b):
        check_selection_invariants(rt.expert_gate[bb], rt.expert_id[bb], cfg.k_a)   # exactly k experts
        for i in range(cfg.n_a):
            check_selection_invariants(rt.patch_gate[bb, i], rt.patch_id[bb, i], cfg.c)  # <= c patches
    # brute force of the whole routing from the definitions
    x = inp.x.astype(np.float64)
    z = x.reshape(cfg.b, -1) @ inp.a_w_expert.astype(np.float64).T
    for bb in range(cfg.b):
        assert rt.expert_id[bb].tolist() == brute_top(z[bb], cfg.k_a)      # softmax is monotone
    gp = np.einsum("bte,ei,tj->bij", x, inp.a_w_b.astype(np.float64), inp.a_w_a.astype(np.float64))
    gd = np.exp(gp) / np.exp(gp).sum(axis=1, keepdims=True)
    np.testing.assert_allclose(rt.patch_gate, gd, rtol=1e-12)
    for bb in range(cfg.b):
        for i in range(cfg.n_a):
            assert rt.patch_id[bb, i].tolist() == brute_top(gd[bb, i], cfg.c)


def test_route_degenerate_modes():
    x = rng(8).standard_normal((2, 12, 4))
    rt = oracle.route(x, n=3, k=3, m=4, c=4)
    assert rt.expert_id.tolist() == [[0, 1, 2]] * 2
    assert rt.patch_id.tolist() == [[[0, 1, 2, 3]] * 3] * 2
    assert np.all(rt.expert_gate == 1.0) and np.all(rt.patch_gate == 1.0)
