"""Pins for the oracle's dynamic capacity (Eq. 15-16) and balance statistics (Eq. 43-44).

Independent checks: a pure-Python brute force that enumerates patches and experts with explicit
comparisons (no argsort), counting identities that follow from Eq. 15 (every patch names exactly k
experts), hand-made cases with known answers.
"""
import math

import numpy as np
import pytest

import oracle


def brute(gp, k):
    b, n, m = gp.shape
    cap, cnts = [], []
    for bb in range(b):
        cnt = [0] * n
        for j in range(m):
            for i in range(n):
                # expert i is among patch j's top-k iff fewer than k experts beat it
                beat = sum(1 for t in range(n) if gp[bb][t][j] > gp[bb][i][j] or (gp[bb][t][j] == gp[bb][i][j] and t < i))
                if beat < k:
                    cnt[i] += 1
        cnts.append(cnt)
        cap.append(max(cnt))
    return np.array(cap), np.array(cnts)


@pytest.mark.parametrize("seed,b,n,m,k", [(0, 3, 5, 7, 2), (1, 2, 4, 9, 1), (2, 4, 8, 16, 3), (3, 1, 6, 6, 6), (4, 2, 3, 1, 2)])
def test_capacity_matches_brute_force(seed, b, n, m, k):
    gp = np.random.default_rng(seed).standard_normal((b, n, m))
    res = oracle.capacity(gp, k)
    cap, cnt = brute(gp, k)
    np.testing.assert_array_equal(res.capacity, cap)
    np.testing.assert_array_equal(res.count, cnt)


def test_counting_identities_and_statistics():
    b, n, m, k = 3, 6, 12, 2
    gp = np.random.default_rng(7).standard_normal((b, n, m))
    res = oracle.capacity(gp, k)
    assert np.all(res.count.sum(axis=1) == m * k)                     # every patch names k experts
    assert np.all(res.capacity >= math.ceil(m * k / n)) and np.all(res.capacity <= m)
    np.testing.assert_allclose(res.load_f.sum(axis=1), n)             # sum_i f_i = n
    np.testing.assert_allclose(res.load_f, n * res.count / (k * m))
    np.testing.assert_allclose(res.load_p.sum(axis=1), 1.0)           # gates are a softmax over experts
    e = np.exp(gp - gp.max(axis=1, keepdims=True))
    np.testing.assert_allclose(res.load_p, (e / e.sum(axis=1, keepdims=True)).mean(axis=2), rtol=1e-12)


def test_known_cases():
    n, m = 4, 8
    # every patch prefers experts in index order: with k = 1 expert 0 gets all m patches
    gp = np.tile(-np.arange(n, dtype=np.float64)[:, None], (1, 1, m))
    assert oracle.capacity(gp, 1).capacity[0] == m
    # exact ties everywhere: the lower indices win, so experts 0..k-1 get every patch
    res = oracle.capacity(np.zeros((1, n, m)), 2)
    np.testing.assert_array_equal(res.count[0], [m, m, 0, 0])
    assert res.capacity[0] == m and np.all(res.margin == 0.0)
    # perfectly balanced: patch j prefers expert j % n -> count m/n each, capacity m/n
    gp = np.full((1, n, m), -5.0)
    for j in range(m):
        gp[0, j % n, j] = 5.0
    res = oracle.capacity(gp, 1)
    np.testing.assert_array_equal(res.count[0], [m // n] * n)
    assert res.capacity[0] == m // n
    np.testing.assert_allclose(res.load_f[0], 1.0)                    # balanced load: f_i = 1
    # k = n: every expert gets every patch
    assert oracle.capacity(np.random.default_rng(1).standard_normal((2, n, m)), n).capacity.tolist() == [m, m]


def test_capacity_bounds_the_fixed_c_selection():
    # with c = capacity, the top-c patches of an expert contain every patch that named it in stage 1
    # whenever that expert's stage-1 patches are also its c best (true when the gate order agrees);
    # what always holds: no expert was named by more than c patches
    gp = np.random.default_rng(11).standard_normal((2, 5, 10))
    res = oracle.capacity(gp, 2)
    assert np.all(res.count.max(axis=1) == res.capacity)


# --------------------------------------------------------------------------- balance loss (Eq. 42)
def test_balance_loss_known_values():
    n, m, alpha = 4, 8, 0.01
    # perfectly even routing: all logits equal -> P_i = 1/n; a rotation of preferences (patch j prefers
    # expert j % n by a hair) -> with k = 1 every expert is named m/n times, f_i = 1: L = alpha * n * (1/n)
    gp = np.zeros((1, n, m))
    for j in range(m):
        gp[0, j % n, j] = 1e-9
    st = oracle.capacity(gp, 1)
    np.testing.assert_allclose(st.load_f[0], 1.0)
    np.testing.assert_allclose(oracle.balance_loss(st.load_f, st.load_p, alpha), [alpha], rtol=1e-8)
    # collapse: every patch is certain of expert 0 -> f_0 = n, P_0 -> 1: L -> alpha * n, the maximum
    gp = np.full((1, n, m), -50.0)
    gp[0, 0, :] = 50.0
    st = oracle.capacity(gp, 1)
    np.testing.assert_allclose(oracle.balance_loss(st.load_f, st.load_p, alpha), [alpha * n], rtol=1e-12)
    # in between, the loss lies between the two (sum_i f_i = n, sum_i P_i = 1, f_i <= n)
    gp = np.random.default_rng(3).standard_normal((5, n, m)) * 3
    st = oracle.capacity(gp, 2)
    lb = oracle.balance_loss(st.load_f, st.load_p, alpha)
    assert np.all(lb > 0) and np.all(lb <= alpha * n / 2 + 1e-12)   # k = 2: f_i <= n/2


def test_balance_loss_gradient_matches_finite_differences():
    """The loss as a function of the gate values g (Eq. 44 inside Eq. 42) with the counts of Eq. 43
    held fixed: perturb single gates, recompute P and the loss from their definitions."""
    b, n, m, k, alpha = 2, 5, 6, 2, 0.3
    gp = np.random.default_rng(11).standard_normal((b, n, m))
    st = oracle.capacity(gp, k)
    g = oracle.patch_gate(gp)
    grad = oracle.balance_loss_grad(st.load_f, alpha, m)
    assert grad.shape == (b, n, m)
    eps = 1e-6
    for bb, i, j in [(0, 0, 0), (1, 3, 5), (0, 4, 2), (1, 1, 1)]:
        def loss(delta):
            gg = g.copy()
            gg[bb, i, j] += delta
            return alpha * np.sum(st.load_f[bb] * gg[bb].mean(axis=1))     # Eq. 42 with Eq. 44 written out
        fd = (loss(eps) - loss(-eps)) / (2 * eps)
        assert abs(fd - grad[bb, i, j]) <= 1e-9
