"""The input generator: shapes, determinism, and bf16 rounding against torch's conversion."""
import numpy as np
import torch

from paper_2503_02495_amd import synth


def test_round_to_bf16_matches_torch_rne():
    r = np.random.default_rng(0)
    a = np.concatenate([r.standard_normal(20000).astype(np.float32) * np.float32(s)
                        for s in (1.0, 0.02, 1e-3, 300.0)])
    # exact ties: mantissa tail 0x8000 with even / odd kept bit
    ties = np.array([0x3F808000, 0x3F818000, 0xBF808000, 0x3F80FFFF, 0x3F800001], np.uint32).view(np.float32)
    a = np.concatenate([a, ties])
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    got = synth.round_to_bf16(a)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    bits = synth.bf16_bits(got)
    back = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(back, got)


def test_configs_and_determinism():
    for name in synth.CONFIG_ORDER:
        c = synth.CONFIGS[name]
        assert c.l % c.m == 0 and 1 <= c.c <= c.m and 1 <= c.k_a <= c.n_a and 1 <= c.k_m <= c.n_m
    c = synth.CONFIGS["tiny"]
    assert (c.b, c.l, c.d, c.l_p, c.l_a, c.tokens) == (2, 64, 64, 8, 16, 128)
    a, b = synth.make_inputs(c), synth.make_inputs(c)
    for f in ("x", "a_w_expert", "a_w_b", "a_w_a", "wq", "wk", "wv", "wo", "m_w_expert", "a_in", "a_out"):
        assert np.array_equal(getattr(a, f), getattr(b, f))
    assert a.x.shape == (2, 64, 64) and a.a_w_expert.shape == (4, 64 * 64) and a.a_w_a.shape == (64, 8)
    assert a.wq.shape == (4, 64, 16) and a.wo.shape == (4, 16, 64) and a.a_in.shape == (4, 64, 64)
    assert abs(float(a.x.std()) - 1.0) < 0.05 and abs(float(a.a_in.std()) - 0.02) < 0.002
    lm = synth.make_inputs(synth.CONFIGS["lm"])
    assert np.array_equal(synth.round_to_bf16(lm.x), lm.x)      # bf16 configs are bf16-exact
    assert lm.noise_a_expert is None
