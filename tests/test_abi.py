"""The C-ABI library loads, exports every symbol the header declares, and turns every bad
argument into an error on the host -- no compute call is made, so this runs without a GPU."""
import ctypes
import os
import re

import pytest

from paper_2310_04361_amd import binding as B

HEADER = os.path.join(os.path.dirname(os.path.dirname(__file__)), "include", "dmoe.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2310_04361_amd import build
        build.build()
    return B.lib()


def _layer(**kw):
    base = dict(d_model=128, n_experts=16, expert_size=16, router_hidden=32, gated=0, act=0,
                dtype=B.DMOE_F32, weight_format=0, w_up=0x1000, w_gate=None, b_up=None, w_down=0x1000,
                b_down=None, r_w1=0x1000, r_b1=None, r_w2=0x1000, r_b2=None, packed=None, w_scales=None)
    base.update(kw)
    return B.DmoeLayerStruct(**base)


def test_exports_match_header(lib):
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(dmoe_[a-z_0-9]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.dmoe_version() >= 100


def test_struct_layout_matches_header():
    # 8 int32 followed by 11 pointers
    assert ctypes.sizeof(B.DmoeLayerStruct) == 8 * 4 + 11 * 8
    assert B.DmoeLayerStruct.w_up.offset == 32 and B.DmoeLayerStruct.packed.offset == 32 + 9 * 8


def test_workspace_sizes(lib):
    n = ctypes.c_size_t(0)
    L = _layer()
    assert lib.dmoe_workspace_bytes(ctypes.byref(L), 128, ctypes.byref(n)) == B.DMOE_OK
    assert n.value >= 128 * 16 * 4 * 2 and n.value % 256 == 0
    small = n.value
    assert lib.dmoe_workspace_bytes(ctypes.byref(L), 4096, ctypes.byref(n)) == B.DMOE_OK
    assert n.value > small
    assert lib.dmoe_workspace_bytes(ctypes.byref(L), 0, ctypes.byref(n)) == B.DMOE_OK
    assert lib.dmoe_workspace_bytes(ctypes.byref(L), -1, ctypes.byref(n)) == B.DMOE_ERR_SHAPE
    assert lib.dmoe_workspace_bytes(ctypes.byref(L), 2 ** 30, ctypes.byref(n)) == B.DMOE_ERR_SHAPE
    assert lib.dmoe_workspace_bytes(None, 1, ctypes.byref(n)) == B.DMOE_ERR_NULL
    assert lib.dmoe_workspace_bytes(ctypes.byref(L), 1, None) == B.DMOE_ERR_NULL
    assert lib.dmoe_select_workspace_bytes(100, 16, ctypes.byref(n)) == B.DMOE_OK and n.value > 0
    assert lib.dmoe_select_workspace_bytes(100, 0, ctypes.byref(n)) == B.DMOE_ERR_SHAPE
    Lb = _layer(dtype=B.DMOE_BF16, expert_size=24)
    assert lib.dmoe_packed_bytes(ctypes.byref(Lb), ctypes.byref(n)) == B.DMOE_OK
    # padded down and up projections (m = 24 -> 32) plus the two router matrices
    assert n.value >= 2 * (16 * 128 * 32 * 2) + 2 * (32 * 128 + 16 * 32) and n.value % 256 == 0
    assert lib.dmoe_packed_bytes(ctypes.byref(L), ctypes.byref(n)) == B.DMOE_OK and n.value == 0


def test_workspace_never_shrinks_as_tokens_grow(lib):
    """A caller may size the workspace once for its largest batch: the requirement must be
    monotone in n_tokens, also across the token counts where the launch shapes change (small-token
    path up to 16, router workgroups per 64-token group at 96 and 192 groups, window tables)."""
    n = ctypes.c_size_t(0)
    shapes = [dict(d_model=768, n_experts=128, expert_size=24, router_hidden=128),
              dict(d_model=2048, n_experts=256, expert_size=64, router_hidden=256, gated=1, w_gate=0x1000),
              dict(d_model=2048, n_experts=2048, expert_size=8, router_hidden=512, gated=1, w_gate=0x1000),
              dict(d_model=256, n_experts=4, expert_size=128, router_hidden=32)]
    for kw in shapes:
        L = _layer(dtype=B.DMOE_BF16, **kw)
        last = 0
        for T in sorted(set(list(range(0, 40)) + list(range(40, 20000, 61)) +
                            [6143, 6144, 6145, 12287, 12288, 12289])):
            assert lib.dmoe_workspace_bytes(ctypes.byref(L), T, ctypes.byref(n)) == B.DMOE_OK
            assert n.value >= last, (kw, T, n.value, last)
            last = n.value


def test_layer_validation(lib):
    n = ctypes.c_size_t(0)
    bad = [
        (_layer(d_model=0), B.DMOE_ERR_SHAPE),
        (_layer(n_experts=-3), B.DMOE_ERR_SHAPE),
        (_layer(dtype=7), B.DMOE_ERR_UNSUPPORTED),
        (_layer(weight_format=2), B.DMOE_ERR_UNSUPPORTED),
        (_layer(weight_format=3), B.DMOE_ERR_UNSUPPORTED),                      # 8-bit formats need bf16
        (_layer(weight_format=4), B.DMOE_ERR_UNSUPPORTED),                      # no such format
        (_layer(weight_format=4, dtype=B.DMOE_BF16), B.DMOE_ERR_UNSUPPORTED),
        (_layer(weight_format=1), B.DMOE_ERR_UNSUPPORTED),                      # 8-bit weights need bf16
        (_layer(weight_format=1, dtype=B.DMOE_BF16), B.DMOE_ERR_NULL),          # ... and scales
        (_layer(gated=2), B.DMOE_ERR_UNSUPPORTED),
    ]
    for L, code in bad:
        assert lib.dmoe_workspace_bytes(ctypes.byref(L), 8, ctypes.byref(n)) == code
        assert lib.dmoe_last_error()


def test_entry_points_reject_bad_arguments_before_launch(lib):
    ws, big = 0x10000, 1 << 40
    x = y = 0x2000
    L = _layer()
    ref = ctypes.byref
    # router
    assert lib.dmoe_router(ref(L), None, 4, 0x3000, None) == B.DMOE_ERR_NULL
    assert lib.dmoe_router(ref(L), x, -1, 0x3000, None) == B.DMOE_ERR_SHAPE
    assert lib.dmoe_router(ref(_layer(r_w1=None)), x, 4, 0x3000, None) == B.DMOE_ERR_NULL
    assert lib.dmoe_router(ref(_layer(router_hidden=0)), x, 4, 0x3000, None) == B.DMOE_ERR_SHAPE
    assert lib.dmoe_router(ref(_layer(dtype=B.DMOE_BF16, router_hidden=48)), x, 4, 0x3000, None) == B.DMOE_ERR_UNSUPPORTED
    assert lib.dmoe_router(ref(L), x, 0, None, None) == B.DMOE_OK          # T = 0: no-op
    # select
    sel = lambda **k: lib.dmoe_select(*[k.get(a, d) for a, d in (
        ("scores", 0x3000), ("T", 8), ("E", 16), ("tau", 0.5), ("mask", None), ("k", None),
        ("counts", None), ("offsets", 0x4000), ("lists", 0x5000), ("ws", ws), ("wsb", big),
        ("stream", None))])
    assert sel(tau=1.5) == B.DMOE_ERR_TAU
    assert sel(tau=-0.01) == B.DMOE_ERR_TAU
    assert sel(tau=float("nan")) == B.DMOE_ERR_TAU
    assert sel(scores=None) == B.DMOE_ERR_NULL
    assert sel(offsets=None) == B.DMOE_ERR_NULL
    assert sel(lists=None) == B.DMOE_ERR_NULL
    assert sel(E=0) == B.DMOE_ERR_SHAPE
    assert sel(T=-2) == B.DMOE_ERR_SHAPE
    assert sel(ws=None) == B.DMOE_ERR_WORKSPACE
    assert sel(ws=ws + 8) == B.DMOE_ERR_WORKSPACE
    assert sel(wsb=16) == B.DMOE_ERR_WORKSPACE
    # expert_ffn
    ffn = lambda L=L, **k: lib.dmoe_expert_ffn(ref(L), *[k.get(a, d) for a, d in (
        ("x", x), ("T", 8), ("offsets", 0x4000), ("lists", 0x5000), ("y", y), ("ws", ws),
        ("wsb", big), ("stream", None))])
    assert ffn(x=None) == B.DMOE_ERR_NULL
    assert ffn(offsets=None) == B.DMOE_ERR_NULL
    assert ffn(wsb=0) == B.DMOE_ERR_WORKSPACE
    assert ffn(L=_layer(act=9)) == B.DMOE_ERR_UNSUPPORTED
    assert ffn(L=_layer(w_down=None)) == B.DMOE_ERR_NULL
    assert ffn(L=_layer(gated=1)) == B.DMOE_ERR_NULL                        # no w_gate
    assert ffn(L=_layer(gated=1, w_gate=0x1000, b_up=0x1000)) == B.DMOE_ERR_UNSUPPORTED
    assert ffn(L=_layer(dtype=B.DMOE_BF16, d_model=256)) == B.DMOE_ERR_NULL            # not packed
    assert ffn(L=_layer(dtype=B.DMOE_BF16, d_model=100, packed=0x1000)) == B.DMOE_ERR_UNSUPPORTED
    assert ffn(L=_layer(dtype=B.DMOE_BF16, d_model=256, expert_size=200, packed=0x1000)) == B.DMOE_ERR_UNSUPPORTED
    assert ffn(L=_layer(dtype=B.DMOE_BF16, d_model=256, expert_size=128, gated=1, w_gate=0x1000,
                        packed=0x1000)) == B.DMOE_ERR_UNSUPPORTED
    assert ffn(T=0, ws=None, wsb=0) == B.DMOE_OK
    # forward
    fwd = lambda L=L, **k: lib.dmoe_forward(ref(L), *[k.get(a, d) for a, d in (
        ("x", x), ("T", 8), ("tau", 0.5), ("y", y), ("scores", None), ("mask", None),
        ("offsets", None), ("lists", None), ("ws", ws), ("wsb", big), ("stream", None))])
    assert fwd(tau=2.0) == B.DMOE_ERR_TAU
    assert fwd(y=None) == B.DMOE_ERR_NULL
    assert fwd(offsets=0x4000) == B.DMOE_ERR_NULL                           # lists missing
    assert fwd(ws=None) == B.DMOE_ERR_WORKSPACE
    assert fwd(L=_layer(r_w2=None)) == B.DMOE_ERR_NULL
    assert fwd(T=0, ws=None, wsb=0) == B.DMOE_OK
    assert b"workspace" in lib.dmoe_last_error() or lib.dmoe_last_error() is not None
    # forward on the library's static workspace: the same checks, and a size limit
    sfw = lambda L=L, **k: lib.dmoe_forward_static(ref(L), *[k.get(a, d) for a, d in (
        ("x", x), ("T", 8), ("tau", ctypes.c_float(0.5)), ("y", y), ("stream", None))])
    assert sfw(tau=ctypes.c_float(2.0)) == B.DMOE_ERR_TAU
    assert sfw(y=None) == B.DMOE_ERR_NULL
    assert sfw(L=_layer(r_w2=None)) == B.DMOE_ERR_NULL
    assert sfw(T=-1) == B.DMOE_ERR_SHAPE
    assert sfw(T=0) == B.DMOE_OK
    assert sfw(T=2 ** 20) == B.DMOE_ERR_WORKSPACE                            # beyond the 32 MiB array
    assert b"static" in lib.dmoe_last_error()
    # pack
    Lb = _layer(dtype=B.DMOE_BF16, d_model=256)
    assert lib.dmoe_pack_weights(ref(Lb), None, 0, None) == B.DMOE_ERR_NULL
    assert lib.dmoe_pack_weights(ref(_layer(dtype=B.DMOE_BF16)), 0x10000, 1 << 30, None) == B.DMOE_ERR_UNSUPPORTED
    assert lib.dmoe_pack_weights(ref(Lb), 0x10000, 16, None) == B.DMOE_ERR_WORKSPACE
    assert lib.dmoe_pack_weights(ref(L), None, 0, None) == B.DMOE_OK          # fp32: no-op
    # a layer with a router is packed with its router: missing router matrices are an error, not
    # a silently unpacked router (router_hidden = 0 declares a layer without one)
    assert lib.dmoe_pack_weights(ref(_layer(dtype=B.DMOE_BF16, d_model=256, r_w1=None)), 0x10000,
                                 1 << 30, None) == B.DMOE_ERR_NULL
    assert lib.dmoe_pack_weights(ref(_layer(dtype=B.DMOE_BF16, d_model=256, r_w2=None)), 0x10000,
                                 1 << 30, None) == B.DMOE_ERR_NULL
    assert lib.dmoe_pack_weights(ref(_layer(dtype=B.DMOE_BF16, d_model=256, router_hidden=48)), 0x10000,
                                 1 << 30, None) == B.DMOE_ERR_UNSUPPORTED
    # timing slots are readable without enabling
    assert lib.dmoe_timing_slots() >= 8
    assert lib.dmoe_timing_read(999, None, None, None) == B.DMOE_ERR_SHAPE


def test_group_calls_reject_bad_arguments_before_launch(lib):
    LP = ctypes.POINTER(B.DmoeLayerStruct)
    a, b = _layer(), _layer()
    other = _layer(n_experts=32)
    n = ctypes.c_size_t(0)
    one = ctypes.c_size_t(0)
    assert lib.dmoe_workspace_bytes(ctypes.byref(a), 128, ctypes.byref(one)) == B.DMOE_OK
    refs = (LP * 2)(ctypes.pointer(a), ctypes.pointer(b))
    assert lib.dmoe_group_workspace_bytes(refs, 2, 128, ctypes.byref(n)) == B.DMOE_OK
    assert n.value == 2 * one.value                  # the sum of the layers' workspaces
    assert lib.dmoe_group_workspace_bytes(refs, 0, 128, ctypes.byref(n)) == B.DMOE_ERR_SHAPE
    assert lib.dmoe_group_workspace_bytes(refs, 5, 128, ctypes.byref(n)) == B.DMOE_ERR_SHAPE
    assert lib.dmoe_group_workspace_bytes(None, 2, 128, ctypes.byref(n)) == B.DMOE_ERR_NULL
    taus = (ctypes.c_float * 2)(0.5, 0.5)
    ys = (ctypes.c_void_p * 2)(0x2000, 0x3000)
    ws = 0x100000
    args = (0x4000, 128, taus, ys, ws, n.value, None)
    mixed = (LP * 2)(ctypes.pointer(a), ctypes.pointer(other))
    assert lib.dmoe_forward_group(mixed, 2, *args) == B.DMOE_ERR_UNSUPPORTED   # two shapes
    assert b"one shape" in lib.dmoe_last_error()
    assert lib.dmoe_forward_group(refs, 0, *args) == B.DMOE_ERR_SHAPE
    assert lib.dmoe_forward_group(refs, 2, 0x4000, 128, None, ys, ws, n.value, None) == B.DMOE_ERR_NULL
    bad_tau = (ctypes.c_float * 2)(0.5, 1.5)
    assert lib.dmoe_forward_group(refs, 2, 0x4000, 128, bad_tau, ys, ws, n.value, None) == B.DMOE_ERR_TAU
    no_y = (ctypes.c_void_p * 2)(0x2000, None)
    assert lib.dmoe_forward_group(refs, 2, 0x4000, 128, taus, no_y, ws, n.value, None) == B.DMOE_ERR_NULL
    assert lib.dmoe_forward_group(refs, 2, 0x4000, 128, taus, ys, ws, n.value - 256, None) == B.DMOE_ERR_WORKSPACE
    assert lib.dmoe_forward_group(refs, 2, None, 0, taus, ys, None, 0, None) == B.DMOE_OK  # no tokens: no-op
