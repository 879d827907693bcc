"""The C-ABI boundary without a GPU: the library loads, exports every symbol the header declares,
and rejects bad arguments on the host before touching any device state (no compute calls here)."""
import ctypes
import os
import re

import pytest

from paper_2503_02495_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # a 16-byte-aligned non-NULL address that is never dereferenced by validation


def header_symbols():
    text = open(os.path.join(ROOT, "include", "uoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(uoe_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    syms = header_symbols()
    assert set(syms) == set(B.EXPORTS)
    L = B.lib()
    for s in syms:
        assert getattr(L, s) is not None


def test_struct_layout_matches_header():
    assert ctypes.sizeof(B.BlockDesc) == 16 * 4
    assert ctypes.sizeof(B.SmhaWeights) == 7 * 8 and ctypes.sizeof(B.UomeWeights) == 5 * 8
    assert ctypes.sizeof(B.RoutingOut) == 4 * 8


def good(**kw):
    base = dict(b=2, l=64, d=64, n=4, k=2, m=8, c=2, width=16, dtype=B.F32,
                flags=B.FLAG_RESIDUAL | B.FLAG_GATE_EXPERT | B.FLAG_GATE_PATCH)
    base.update(kw)
    return B.block_desc(**base)


def test_status_strings():
    assert B.status_string(B.OK) == "ok"
    for s in (1, 2, 3, 4, 99):
        assert isinstance(B.status_string(s), str) and B.status_string(s)


def test_workspace_bytes():
    a = B.workspace_bytes(good(), None)
    m = B.workspace_bytes(None, good(m=1, c=1, width=64))
    both = B.workspace_bytes(good(), good(m=1, c=1, width=64))
    assert a > 0 and m > 0 and both >= a + m
    assert B.workspace_bytes(good(l=63), None) == 0       # invalid descriptor -> 0
    assert B.workspace_bytes(None, None) == 0


@pytest.mark.parametrize("kw,want", [
    (dict(l=63), B.ERR_INVALID_ARG),             # l % m != 0
    (dict(k=5), B.ERR_INVALID_ARG),              # k > n
    (dict(c=9), B.ERR_INVALID_ARG),              # c > m
    (dict(c=0), B.ERR_INVALID_ARG),
    (dict(b=0), B.ERR_INVALID_ARG),
    (dict(dtype=7), B.ERR_INVALID_ARG),
    (dict(flags=1 << 9), B.ERR_INVALID_ARG),
    (dict(rope_dim=3), B.ERR_INVALID_ARG),       # odd
    (dict(rope_dim=18), B.ERR_INVALID_ARG),      # > width
    (dict(d=60), B.ERR_UNSUPPORTED),             # d % 8 != 0
    (dict(width=12), B.ERR_UNSUPPORTED),
    (dict(n=33, k=2), B.ERR_UNSUPPORTED),
])
def test_descriptor_validation(kw, want):
    d = good(**kw)
    args = [FAKE] * 10
    assert B.route(d, *args, FAKE, stream=0, check=False, ws_bytes=1 << 30) == want
    assert B.smha_forward(d, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE + 16, FAKE,
                          stream=0, check=False, ws_bytes=1 << 30) == want


def test_causal_and_rope_belong_to_the_attention_block():
    for kw in (dict(flags=B.FLAG_CAUSAL), dict(rope_dim=8)):
        d = good(**kw)
        # routing ignores them (same descriptor serves uoe_route and uoe_smha_forward)
        assert B.route(d, *([FAKE] * 10), FAKE, stream=0, check=False, ws_bytes=8) == B.ERR_WORKSPACE
        u = good(m=1, c=1, width=64, **kw)
        assert B.uome_forward(u, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE + 16, FAKE, stream=0, check=False,
                              ws_bytes=1 << 30) == B.ERR_UNSUPPORTED
        # accepted by the attention call (fails later, on the too-small workspace)
        assert B.smha_forward(d, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE + 16, FAKE, stream=0,
                              check=False, ws_bytes=8) == B.ERR_WORKSPACE
        assert B.smha_forward_masked(d, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE + 16, FAKE,
                                     stream=0, check=False, ws_bytes=8) == B.ERR_WORKSPACE


def test_route_capacity_argument_validation():
    d = good()
    big = 1 << 30
    call = lambda *a, **k: B.route_capacity(d, *a, stream=0, check=False, **k)
    assert call(FAKE, FAKE, FAKE, None, 2, FAKE, None, None, FAKE, ws_bytes=16) == B.ERR_WORKSPACE    # accepted
    assert call(FAKE, None, FAKE, None, 2, FAKE, None, None, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # no data router
    assert call(FAKE, FAKE, FAKE, None, 0, FAKE, None, None, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # patch_k < 1
    assert call(FAKE, FAKE, FAKE, None, 5, FAKE, None, None, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # patch_k > n
    assert call(FAKE, FAKE, FAKE, None, 2, None, None, None, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # no output
    wide = good(n=32, k=2, m=512, c=2, l=512)
    assert B.route_capacity(wide, FAKE, FAKE, FAKE, None, 2, FAKE, None, None, FAKE, stream=0, check=False,
                            ws_bytes=big) == B.ERR_UNSUPPORTED                                        # n*m logits > LDS stage


def test_reserved_fields_must_be_zero():
    d = good()
    d.reserved[2] = 1
    assert B.route(d, *([FAKE] * 10), FAKE, stream=0, check=False, ws_bytes=1 << 30) == B.ERR_INVALID_ARG


def test_route_argument_validation():
    d = good()
    big = 1 << 30
    call = lambda *a, **k: B.route(d, *a, stream=0, check=False, **k)
    outs = [FAKE] * 4
    assert call(None, FAKE, FAKE, FAKE, None, None, *outs, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # x NULL
    assert call(FAKE + 2, FAKE, FAKE, FAKE, None, None, *outs, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # misaligned
    assert call(FAKE, FAKE, FAKE, None, None, None, *outs, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # w_a without w_b
    assert call(FAKE, None, FAKE, FAKE, None, None, *outs, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # no w_expert, k<n
    assert call(FAKE, FAKE, None, None, None, None, *outs, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # no data router, c<m
    assert call(FAKE, FAKE, FAKE, FAKE, None, None, *outs, None, ws_bytes=big) == B.ERR_WORKSPACE
    assert call(FAKE, FAKE, FAKE, FAKE, None, None, *outs, FAKE, ws_bytes=16) == B.ERR_WORKSPACE
    with pytest.raises(B.UoeError) as e:
        B.route(d, None, FAKE, FAKE, FAKE, None, None, *outs, FAKE, stream=0, ws_bytes=big)
    assert e.value.status == B.ERR_INVALID_ARG


def test_smha_uome_layer_argument_validation():
    d = good()
    big = 1 << 30
    sm = lambda *a, **k: B.smha_forward(d, *a, stream=0, check=False, **k)
    assert sm(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # out aliases x
    assert sm(FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE + 16, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # wo NULL
    assert sm(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE + 16, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # gate flag, no gate
    assert sm(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE + 16, FAKE, ws_bytes=8) == B.ERR_WORKSPACE

    u = good(m=1, c=1, width=64, flags=B.FLAG_RESIDUAL | B.FLAG_GATE_EXPERT)
    um = lambda desc, *a, **k: B.uome_forward(desc, *a, stream=0, check=False, **k)
    assert um(u, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # out aliases u
    assert um(u, FAKE, FAKE, FAKE, FAKE, None, None, None, FAKE + 16, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # gate missing
    assert um(u, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE + 16, FAKE, ws_bytes=8) == B.ERR_WORKSPACE
    ds = good(m=8, c=2, width=64, flags=B.FLAG_RESIDUAL)                    # data-selection UoME
    assert um(ds, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE + 16, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # c < m, no patch_idx
    assert um(ds, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE + 16, FAKE, ws_bytes=8) == B.ERR_WORKSPACE      # accepted
    dsg = good(m=8, c=2, width=64, flags=B.FLAG_RESIDUAL | B.FLAG_GATE_PATCH)
    assert um(dsg, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE + 16, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # patch gate missing
    assert um(dsg, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE + 16, FAKE, ws_bytes=8) == B.ERR_WORKSPACE
    ug = good(m=1, c=1, width=64, flags=B.FLAG_RESIDUAL | B.FLAG_GATE_PATCH)
    assert um(ug, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE + 16, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # patch gate flag, no patches

    wa = B.smha_weights(*([FAKE] * 7))
    wm = B.uome_weights(FAKE, FAKE, FAKE)
    ly = lambda a, m_, x, out, **k: B.layer_forward(a, wa, None, None, m_, wm, None, x, out, None, None, FAKE,
                                                    stream=0, check=False, **k)
    assert ly(d, u, FAKE, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG                      # out aliases x
    assert ly(d, good(b=3, m=1, c=1, width=64), FAKE, FAKE + 16, ws_bytes=big) == B.ERR_INVALID_ARG  # b mismatch
    assert ly(d, u, FAKE, FAKE + 16, ws_bytes=64) == B.ERR_WORKSPACE
    lym = lambda a, m_, x, out, **k: B.layer_forward_masked(a, wa, None, None, m_, wm, None, x, FAKE + 32, out, None, None,
                                                            FAKE, stream=0, check=False, **k)
    assert lym(d, u, FAKE, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG                     # the same rules with a padding mask
    assert lym(d, u, FAKE, FAKE + 16, ws_bytes=64) == B.ERR_WORKSPACE
    assert B.balance_loss(d, None, FAKE, 0.01, FAKE, None, stream=0, check=False) == B.ERR_INVALID_ARG   # no statistics
    assert B.balance_loss(d, FAKE, FAKE, 0.01, None, None, stream=0, check=False) == B.ERR_INVALID_ARG   # nothing to write
    assert B.balance_loss(d, FAKE, None, 0.01, FAKE, None, stream=0, check=False) == B.ERR_INVALID_ARG   # the loss needs P
    assert B.balance_loss(d, FAKE, FAKE, float("nan"), FAKE, None, stream=0, check=False) == B.ERR_INVALID_ARG
    assert B.gather(d, FAKE, FAKE, FAKE, FAKE, stream=0, check=False) == B.ERR_INVALID_ARG   # h aliases x
    assert B.gather(d, None, FAKE, FAKE, FAKE, stream=0, check=False) == B.ERR_INVALID_ARG


def test_backward_argument_validation():
    """The backward entry points: unsupported shapes give a zero workspace size and
    UOE_ERR_UNSUPPORTED, bad pointer combinations UOE_ERR_INVALID_ARG, all before any launch.  Shapes
    off the matrix-core grid and fp32 storage are taken by the vector-ALU path, except the UoME block
    with patch-wise data selection."""
    assert ctypes.sizeof(B.SmhaWeightGrads) == 4 * 8 and ctypes.sizeof(B.RouterGrads) == 3 * 8
    big = 1 << 40
    fl = B.FLAG_RESIDUAL | B.FLAG_GATE_EXPERT
    # UoME backward, expert-selection mode: every shape and both storage types
    u = B.block_desc(2, 64, 64, 4, 2, 1, 1, 64, B.BF16, fl)
    assert B.uome_backward_workspace_bytes(u) > 0
    # vector-ALU path (fp32 storage): Z/H and dH/dZ in fp32, plus the weight gradients' partial tiles, here
    # 4 ranges of (sample, slot) pairs (b * k = 4 caps the 8 that so few tiles would ask for)
    assert B.uome_backward_workspace_bytes(B.block_desc(2, 64, 64, 4, 2, 1, 1, 64, B.F32, fl)) == \
        2 * (2 * 64 * 2 * 64 * 4) + 2 * 4 * 4 * 64 * 64 * 4
    assert B.uome_backward_workspace_bytes(B.block_desc(2, 48, 64, 4, 2, 1, 1, 64, B.BF16, fl)) == \
        2 * (2 * 48 * 2 * 64 * 4) + 2 * 4 * 4 * 64 * 64 * 4
    ub = lambda *a, **k: B.uome_backward(u, *a, stream=0, check=False, **k)
    ok = [FAKE, FAKE + 16, FAKE + 32, FAKE, FAKE, None, None, FAKE + 48, FAKE + 64, FAKE + 80, FAKE + 96, FAKE, None, FAKE]
    assert ub(*ok, ws_bytes=8) == B.ERR_WORKSPACE
    bad = list(ok); bad[4] = None                       # gate flag without gates
    assert ub(*bad, ws_bytes=big) == B.ERR_INVALID_ARG
    bad = list(ok); bad[8] = ok[0]                      # d_u aliases u
    assert ub(*bad, ws_bytes=big) == B.ERR_INVALID_ARG
    bad = list(ok); bad[5] = FAKE                       # patch indices on an expert-selection descriptor
    assert ub(*bad, ws_bytes=big) == B.ERR_INVALID_ARG
    uds = B.block_desc(2, 128, 64, 4, 2, 4, 2, 64, B.BF16, fl | B.FLAG_GATE_PATCH)     # data selection, l_p = 32
    assert B.uome_backward_workspace_bytes(uds) > 0
    assert B.uome_backward_workspace_bytes(B.block_desc(2, 128, 64, 4, 2, 8, 2, 64, B.BF16, fl)) == 0    # l_p = 16
    assert B.uome_backward_workspace_bytes(B.block_desc(2, 128, 64, 4, 2, 4, 2, 64, B.F32, fl)) == 0     # fp32 storage
    dsb = lambda *a, **k: B.uome_backward(uds, *a, stream=0, check=False, **k)
    okd = list(ok); okd[5] = FAKE; okd[6] = FAKE; okd[12] = FAKE
    assert dsb(*okd, ws_bytes=8) == B.ERR_WORKSPACE
    bad = list(okd); bad[5] = None                      # c < m needs patch indices
    assert dsb(*bad, ws_bytes=big) == B.ERR_INVALID_ARG
    bad = list(okd); bad[6] = None                      # patch gate flag without patch gates
    assert dsb(*bad, ws_bytes=big) == B.ERR_INVALID_ARG
    # SMHA backward: every shape and both storage types (d_h in {32, 64, 128} with l_p a multiple of 32 on the
    # matrix cores, the rest on the vector ALU, whose [units, l_a, l_a] arrays bound the size)
    a = B.block_desc(2, 128, 64, 4, 2, 4, 2, 32, B.BF16, fl | B.FLAG_GATE_PATCH)
    assert B.smha_backward_workspace_bytes(a) > 0
    assert B.smha_backward_workspace_bytes(B.block_desc(2, 128, 64, 4, 2, 8, 2, 32, B.BF16, fl)) > 0    # l_p = 16
    assert B.smha_backward_workspace_bytes(B.block_desc(2, 128, 64, 4, 2, 4, 2, 16, B.F32, fl)) > 0     # d_h = 16, fp32
    assert B.smha_backward_workspace_bytes(B.block_desc(64, 8192, 64, 4, 4, 8, 8, 16, B.F32, fl)) == 0  # 256 units of 8192 rows
    wa = B.smha_weights(*([FAKE] * 7))
    dw = B.smha_weight_grads(FAKE + 16, FAKE + 32, FAKE + 48, FAKE + 64)
    sb = lambda *args, **k: B.smha_backward(a, *args, stream=0, check=False, **k)
    assert sb(FAKE, wa, FAKE, FAKE, FAKE, FAKE, None, FAKE + 16, FAKE + 32, dw, None, None, FAKE, ws_bytes=8) == B.ERR_WORKSPACE
    assert sb(FAKE, wa, FAKE, FAKE, FAKE, None, None, FAKE + 16, FAKE + 32, dw, None, None, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG
    assert sb(FAKE, wa, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE + 16, FAKE, dw, None, None, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG  # d_x aliases x
    # router backward: at least one router, w_b and w_a together, gates with their routers
    rb = lambda *args, **k: B.route_backward(a, *args, stream=0, check=False, **k)
    assert B.route_backward_workspace_bytes(a) > 0
    assert rb(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE + 16, FAKE, FAKE, FAKE, FAKE, ws_bytes=8) == B.ERR_WORKSPACE
    assert rb(FAKE, None, None, None, None, None, None, None, FAKE + 16, None, None, None, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG
    assert rb(FAKE, None, FAKE, None, None, FAKE, None, FAKE, FAKE + 16, None, FAKE, FAKE, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG
    assert rb(FAKE, FAKE, None, None, None, None, FAKE, None, FAKE + 16, FAKE, None, None, FAKE, ws_bytes=big) == B.ERR_INVALID_ARG
    # layer backward: the sizes of its parts, the same shape rules
    assert B.layer_backward_workspace_bytes(a, u) == 0              # l differs (128 vs 64)
    u2 = B.block_desc(2, 128, 64, 4, 2, 1, 1, 64, B.BF16, fl)
    need = B.layer_backward_workspace_bytes(a, u2)
    assert need >= max(B.smha_backward_workspace_bytes(a), B.uome_backward_workspace_bytes(u2))
    wm = B.uome_weights(FAKE, FAKE, FAKE)
    ra = B.routing_out(FAKE, FAKE, FAKE, FAKE)
    rm = B.routing_out(FAKE, FAKE)
    lb = lambda dra, drm, **k: B.layer_backward(a, wa, u2, wm, FAKE, None, ra, rm, FAKE + 16, FAKE + 32, dw, dra,
                                                FAKE + 48, FAKE + 64, drm, FAKE, stream=0, check=False, **k)
    assert lb(B.router_grads(FAKE, FAKE, FAKE), B.router_grads(FAKE), ws_bytes=8) == B.ERR_WORKSPACE
    assert lb(None, B.router_grads(FAKE), ws_bytes=big) == B.ERR_INVALID_ARG      # SMHA has routers, no place for their gradients
    lbm = lambda dra, drm, **k: B.layer_backward_masked(a, wa, u2, wm, FAKE, FAKE + 80, None, ra, rm, FAKE + 16, FAKE + 32,
                                                        dw, dra, FAKE + 48, FAKE + 64, drm, FAKE, stream=0, check=False, **k)
    assert lbm(B.router_grads(FAKE, FAKE, FAKE), B.router_grads(FAKE), ws_bytes=8) == B.ERR_WORKSPACE
    assert lbm(None, B.router_grads(FAKE), ws_bytes=big) == B.ERR_INVALID_ARG
