"""Pins for the oracle's optional SMHA features: shared causal mask and gathered padding mask
(Sec. III-C.3, Eq. 41, Fig. 4) and partial RoPE (Eq. 32).  Independent references are NumPy
formulations (explicitly gathered masks, complex-number rotation), not the oracle."""
import numpy as np
import pytest

import oracle

R, GE, GP, CA = oracle.RESIDUAL, oracle.GATE_EXPERT, oracle.GATE_PATCH, oracle.CAUSAL


def rng(seed=0):
    return np.random.default_rng(seed)


def masked_softmax(s, ok):
    s = np.where(ok, s, -np.inf)
    mx = np.max(s, axis=-1, keepdims=True)
    mx = np.where(np.isfinite(mx), mx, 0.0)
    e = np.where(ok, np.exp(s - mx), 0.0)
    den = e.sum(axis=-1, keepdims=True)
    return np.where(den > 0, e / np.where(den > 0, den, 1.0), 0.0)


def rope_complex(v, rope_dim):
    """Rotate the last rope_dim dims of rows of v [rows, d_h]; row r at position r; complex form."""
    rows, d_h = v.shape
    out = v.copy()
    if rope_dim == 0:
        return out
    z = v[:, d_h - rope_dim::2] + 1j * v[:, d_h - rope_dim + 1::2]          # pairs (2i, 2i+1)
    theta = 10000.0 ** (-2.0 * np.arange(rope_dim // 2) / rope_dim)
    z = z * np.exp(1j * np.arange(rows)[:, None] * theta[None, :])
    out[:, d_h - rope_dim::2] = z.real
    out[:, d_h - rope_dim + 1::2] = z.imag
    return out


def brute(x, wq, wk, wv, wo, eid, pid, m, causal=False, rope_dim=0, pad=None, full_mask=None):
    """Definition with explicit token lists; the causal mask is GATHERED from the full l x l mask
    with the token indices (what Sec. III-C.3 says one would have to do without the shared mask)."""
    b, l, d = x.shape
    l_p = l // m
    d_h = wq.shape[2]
    out = x.copy()
    for bb in range(b):
        for i in eid[bb]:
            toks = np.concatenate([np.arange(p * l_p, (p + 1) * l_p) for p in pid[bb, i]])
            h = x[bb, toks]
            q, k, v = rope_complex(h @ wq[i], rope_dim), rope_complex(h @ wk[i], rope_dim), h @ wv[i]
            ok = np.ones((len(toks), len(toks)), bool)
            if causal:
                ok &= full_mask[np.ix_(toks, toks)]
            if pad is not None:
                ok &= pad[bb, toks].astype(bool)[None, :]
            s = masked_softmax(q @ k.T / np.sqrt(d_h), ok)
            np.add.at(out[bb], toks, s @ v @ wo[i])
    return out


def setup(seed, b=2, d=6, n=3, d_h=6, m=5, c=3, l_p=2, k=2):
    r = rng(seed)
    l = m * l_p
    x = r.standard_normal((b, l, d))
    w = [r.standard_normal((n, d, d_h)) * 0.4 for _ in range(3)] + [r.standard_normal((n, d_h, d)) * 0.4]
    eid = np.stack([np.sort(r.choice(n, k, replace=False)) for _ in range(b)]).astype(np.int32)
    pid = np.stack([[np.sort(r.choice(m, c, replace=False)) for _ in range(n)] for _ in range(b)]).astype(np.int32)
    return r, x, w, eid, pid, np.ones((b, n)), np.ones((b, n, m)), m, l


def test_gathered_causal_mask_is_the_leading_block():
    """Fig. 4: indexing the l x l causal mask with the same ascending indices on both axes gives the
    l_a x l_a lower-triangular matrix, whatever the indices."""
    r = rng(0)
    l = 40
    full = np.tril(np.ones((l, l), bool))
    for _ in range(20):
        toks = np.sort(r.choice(l, 11, replace=False))
        assert np.array_equal(full[np.ix_(toks, toks)], np.tril(np.ones((11, 11), bool)))


@pytest.mark.parametrize("seed", [1, 2])
def test_causal_matches_gathered_mask(seed):
    r, x, w, eid, pid, ge, gd, m, l = setup(seed)
    full = np.tril(np.ones((l, l), bool))
    got = oracle.smha(x, *w, eid, ge, pid, gd, m, flags=R | CA)
    np.testing.assert_allclose(got, brute(x, *w, eid, pid, m, causal=True, full_mask=full), rtol=1e-11, atol=1e-12)
    assert not np.allclose(got, oracle.smha(x, *w, eid, ge, pid, gd, m, flags=R))
    # first selected token of every unit sees only itself: softmax of one score is 1
    b, d_h = x.shape[0], w[0].shape[2]
    l_p = l // m
    single = oracle.smha(x, *w, eid[:, :1], ge, pid, gd, m, flags=CA)
    for bb in range(b):
        i = eid[bb, 0]
        t = pid[bb, i, 0] * l_p
        np.testing.assert_allclose(single[bb, t], x[bb, t] @ w[2][i] @ w[3][i], rtol=1e-11, atol=1e-13)


def test_full_selection_causal_equals_dense_causal_mha():
    r = rng(3)
    b, l, d, n, d_h, m = 2, 10, 6, 2, 4, 5
    x = r.standard_normal((b, l, d))
    w = [r.standard_normal((n, d, d_h)) * 0.4 for _ in range(3)] + [r.standard_normal((n, d_h, d)) * 0.4]
    eid = np.tile(np.arange(n, dtype=np.int32), (b, 1))
    pid = np.tile(np.arange(m, dtype=np.int32), (b, n, 1))
    got = oracle.smha(x, *w, eid, np.ones((b, n)), pid, np.ones((b, n, m)), m, flags=R | CA)
    want = x.copy()
    ok = np.tril(np.ones((l, l), bool))
    for bb in range(b):
        for h in range(n):
            s = masked_softmax((x[bb] @ w[0][h]) @ (x[bb] @ w[1][h]).T / np.sqrt(d_h), ok)
            want[bb] += s @ (x[bb] @ w[2][h]) @ w[3][h]
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)


def test_padding_mask():
    r, x, w, eid, pid, ge, gd, m, l = setup(4)
    b = x.shape[0]
    pad = (r.random((b, l)) > 0.3).astype(np.uint8)
    full = np.tril(np.ones((l, l), bool))
    for causal in (False, True):
        fl = R | (CA if causal else 0)
        got = oracle.smha(x, *w, eid, ge, pid, gd, m, flags=fl, pad_mask=pad)
        np.testing.assert_allclose(got, brute(x, *w, eid, pid, m, causal=causal, pad=pad, full_mask=full),
                                   rtol=1e-11, atol=1e-12)
    # all ones == no mask; all zeros == nothing contributes
    np.testing.assert_array_equal(oracle.smha(x, *w, eid, ge, pid, gd, m, flags=R, pad_mask=np.ones((b, l))),
                                  oracle.smha(x, *w, eid, ge, pid, gd, m, flags=R))
    np.testing.assert_array_equal(oracle.smha(x, *w, eid, ge, pid, gd, m, flags=R, pad_mask=np.zeros((b, l))), x)
    # a padded key changes nothing when its value is changed
    x2 = x.copy()
    x2[pad == 0] += 5.0
    a = oracle.smha(x, *w, eid, ge, pid, gd, m, flags=0, pad_mask=pad)
    c = oracle.smha(x2, *w, eid, ge, pid, gd, m, flags=0, pad_mask=pad)
    np.testing.assert_allclose(a[pad == 1], c[pad == 1], rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("rope_dim", [2, 4, 6])
def test_rope_matches_complex_rotation(rope_dim):
    r, x, w, eid, pid, ge, gd, m, l = setup(5)
    full = np.tril(np.ones((l, l), bool))
    got = oracle.smha(x, *w, eid, ge, pid, gd, m, flags=R | CA, rope_dim=rope_dim)
    want = brute(x, *w, eid, pid, m, causal=True, rope_dim=rope_dim, full_mask=full)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)
    assert not np.allclose(got, oracle.smha(x, *w, eid, ge, pid, gd, m, flags=R | CA))
    np.testing.assert_array_equal(oracle.smha(x, *w, eid, ge, pid, gd, m, flags=R, rope_dim=0),
                                  oracle.smha(x, *w, eid, ge, pid, gd, m, flags=R))


def test_rope_scores_depend_on_relative_position_only():
    """With the whole head rotary, shifting every position by the same amount leaves attention
    unchanged: selecting patches {1,2,3} or {0,1,2,3} changes compacted positions by one patch, so a
    unit built from identical tokens must give identical rows for the shared tokens when the extra
    leading patch is masked out as padding."""
    r = rng(6)
    b, d, n, d_h, m, l_p = 1, 4, 1, 4, 4, 2
    l = m * l_p
    x = r.standard_normal((b, l, d))
    w = [r.standard_normal((n, d, d_h)) * 0.5 for _ in range(3)] + [r.standard_normal((n, d_h, d)) * 0.5]
    eid = np.zeros((1, 1), np.int32)
    ge, gd = np.ones((1, 1)), np.ones((1, 1, m))
    a = oracle.smha(x, *w, eid, ge, np.array([[[1, 2, 3]]], np.int32), gd, m, flags=0, rope_dim=4)
    pad = np.ones((1, l), np.uint8)
    pad[0, :l_p] = 0                      # the extra leading patch is padding: keys ignored
    c = oracle.smha(x, *w, eid, ge, np.array([[[0, 1, 2, 3]]], np.int32), gd, m, flags=0, rope_dim=4, pad_mask=pad)
    np.testing.assert_allclose(a[0, l_p:], c[0, l_p:], rtol=1e-10, atol=1e-12)
