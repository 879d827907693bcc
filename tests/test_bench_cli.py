"""Host-side contract of bench.py that needs no GPU: more than one GPU is refused with a message,
and the FLOP model counts what the descriptor says."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_flop_model():
    sys.path.insert(0, ROOT)
    import dataclasses

    import bench
    from paper_2503_02495_amd import synth

    c = synth.CONFIGS["lm"]
    fl = bench.layer_flops(c)
    assert fl["uome"] == 4 * c.b * c.k_m * c.l * c.d * c.d_e               # two GEMMs, 2 FLOP per MAC
    assert fl["qkv"] == 3 * 2 * c.b * c.k_a * c.l_a * c.d * c.d_h
    assert fl["total"] == sum(v for k, v in fl.items() if k != "total")
    half = dataclasses.replace(c, m_m=16, c_m=8)                            # data-selected UoME: half the rows
    assert bench.layer_flops(half)["uome"] * 2 == fl["uome"]
    assert "m16 c8" in bench.describe(half) and "m16 c8" not in bench.describe(c).split("UoME")[1]
