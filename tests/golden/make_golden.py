"""Writes tests/golden/tiny_layer.json from the CPU oracle alone (never from the GPU path).

    python tests/golden/make_golden.py

The paper prints no worked numeric example of the layer, so this fixture is a regression pin of the
oracle on the tiny fp32 workload (seed 0): the routing indices, and a few output values, as the
oracle computed them when its pins (tests/test_oracle_*.py) were green.  A later change to the
oracle's arithmetic that moves these values must say which passage of the paper justifies it.
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
from paper_2503_02495_amd import synth  # noqa: E402


def main():
    cfg = synth.CONFIGS["tiny"]
    inp = synth.make_inputs(cfg)
    res = oracle.layer_forward(inp, oracle.RESIDUAL | oracle.GATE_EXPERT | oracle.GATE_PATCH,
                               oracle.RESIDUAL | oracle.GATE_EXPERT)
    pick = [(0, 0, 0), (0, 17, 5), (1, 40, 63), (1, 63, 31)]
    fixture = {
        "workload": "tiny, seed 0, flags: residual + expert gate + patch gate",
        "smha_expert_id": res.routing_a.expert_id.tolist(),
        "smha_patch_id": res.routing_a.patch_id.tolist(),
        "uome_expert_id": res.routing_m.expert_id.tolist(),
        "smha_expert_gate_sample0": [float("%.12e" % v) for v in res.routing_a.expert_gate[0]],
        "out_at": [[list(p), float("%.12e" % res.out[p])] for p in pick],
        "out_minus_x_abs_sum": float("%.10e" % np.abs(res.out - inp.x).sum()),
    }
    with open(os.path.join(HERE, "tiny_layer.json"), "w") as f:
        json.dump(fixture, f, indent=1)
    print("wrote tiny_layer.json")


if __name__ == "__main__":
    main()
