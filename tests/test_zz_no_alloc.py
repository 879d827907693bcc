"""uoe_route_static, the entry point that allocates nothing (its scratch is a fixed array in the
library image), against uoe_route on the same inputs: same kernels in the same order, so indices and
gates must be bit-identical.  Two calls in a row, the second with a smaller input (the shared scratch
keeps the first call's contents), then the first shape again."""
import pytest
import torch

from paper_2503_02495_amd import binding as B
from paper_2503_02495_amd import synth
from paper_2503_02495_amd.harness import DeviceLayer

pytestmark = pytest.mark.gpu


def route_both_ways(cfg, w_std):
    inp = synth.make_inputs(cfg, w_std=w_std)
    dev = DeviceLayer(inp, B.FLAG_RESIDUAL, B.FLAG_RESIDUAL)
    dev.route_a()                                   # uoe_route with the caller's workspace
    torch.cuda.synchronize()
    want = [t.clone() for t in (dev.a_expert_idx, dev.a_expert_gate, dev.a_patch_idx, dev.a_patch_gate)]
    got = [torch.full_like(t, -1) for t in want]
    B.route_static(dev.smha, dev.x, dev.a_w_expert, dev.a_w_b, dev.a_w_a, dev.noise_a_expert, dev.noise_a_patch, *got)
    torch.cuda.synchronize()
    for name, g, w in zip(("expert_idx", "expert_gate", "patch_idx", "patch_gate"), got, want):
        assert torch.equal(g.view(torch.int32), w.view(torch.int32)), (cfg.name, name)


def test_route_static_matches_route_on_two_calls_in_a_row():
    big = synth.CONFIGS["longrange"]                 # 2.2 MiB of partial sums
    small = synth.small_config(b=3, l=140, d=64, n_a=4, d_h=32, m=10, c=3, k_a=3, n_m=4, d_e=64, k_m=2, dtype=synth.BF16)
    print("route_static longrange", flush=True)
    route_both_ways(big, 0.02)
    print("route_static small bf16 shape", flush=True)
    route_both_ways(small, 0.06)
    print("route_static tiny fp32 shape", flush=True)
    route_both_ways(synth.CONFIGS["tiny"], 0.02)
    print("route_static longrange again", flush=True)
    route_both_ways(big, 0.02)


def test_route_static_rejects_a_request_beyond_its_scratch():
    # 64 data-router chunks x b 128 x n 32 x m 256 fp32 partial sums = 268 MB: rejected on the host
    blk = B.block_desc(128, 4096, 64, 32, 2, 256, 2, 16, B.BF16, 0)
    fake = 0x10000
    st = B.route_static(blk, fake, fake, fake, fake, None, None, fake, fake, fake, fake, stream=0, check=False)
    assert st == B.ERR_SCRATCH_LIMIT
    assert "scratch" in B.status_string(st)
