"""Fully 8-bit layers (weight format DMOE_W_FP8_E4M3_A8, the lower-precision layers of Appendix C):
8-bit expert weights, 8-bit expert inputs and 8-bit hidden activations -- every selected
(token, expert) row of hidden activations is rounded to bf16 and then quantised to E4M3 with a
power-of-two row scale before the down-projection.  The oracle applies the same two quantisers
(oracle.quantize_rows_e4m3 on the input, expert_ffn(..., quantize_h=True)) around its fp64
experts.  H rows of 64 neurons run the 8-bit matrix-core down-projection; other sizes quantise H
in place and keep their bf16 kernels; every batch size takes the list-based kernels."""
import numpy as np
import pytest

from helpers import (TOL, check_fully_8bit, lists_from_mask, oracle_ffn, small_cfg,
                     tokenwise_rel_err)
from paper_2310_04361_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2310_04361_amd import binding
    binding.lib()
    return binding


def _a8_layer(cfg, seed):
    layer = wl.quantize_experts_e4m3(wl.make_layer(cfg, seed))
    layer["x8"] = True
    layer["a8"] = True
    return layer


def _oracle_a8(oracle, layer, x, mask):
    xq, _ = oracle.quantize_rows_e4m3(x)
    return oracle_ffn(oracle, layer, xq, mask, quantize_h=True)


def _check(oracle, layer, x, mask, got, dtype):
    """Against the oracle, to the bar of helpers.check_fully_8bit."""
    xq, _ = oracle.quantize_rows_e4m3(x)
    ref = oracle_ffn(oracle, layer, xq, mask, quantize_h=True)
    return check_fully_8bit(oracle, layer, xq, mask, got, ref, TOL[dtype])


# 8-bit down-projection: gated experts of 64 (ragged token counts, expert counts that are not a
# multiple of the four-unit rotation or of the 32-expert mask batch), experts of 48 in rows of
# 64, plain experts of 64, plain experts of 128 (two units of 64 per expert); in-place
# quantisation + bf16 kernels: rows of 32, one-tile experts; batches of at most 16 tokens
SHAPES = [("cfg4", 300, 16), ("cfg4", 700, 8), ("cfg4", 129, 37), ("cfg4", 1000, 70), ("cfg4", 17, 16),
          ("cfg4", 16, 64), ("cfg4", 5, 16), ("cfg4", 1, 16), ("cfg4", 200, 600), ("cfg4", 70, 1),
          ("cfg2", 300, 32), ("paper", 260, 8), ("paper", 1000, None), ("paper", 130, 37), ("paper", 9, 5), ("gemma_paper", 200, 64), ("cfg5b", 9, None)]


@pytest.mark.parametrize("name,T,E", SHAPES)
def test_forward_fully_8bit(B, oracle, name, T, E):
    import torch
    cfg = small_cfg(name, T, E)
    print(f"fully 8-bit {name} T={T} E={cfg.E}", flush=True)
    layer = _a8_layer(cfg, 3)
    x = wl.make_input(cfg, 3)
    L = B.Layer(layer, cfg.dtype)
    tau = float(np.float32(0.4))
    xd = B.to_device(x, cfg.dtype)
    y, ex = B.dmoe_forward(L, xd, tau, want_scores=True, want_mask=True)
    torch.cuda.synchronize()
    mask, _ = oracle.select(ex["scores"].cpu().numpy().astype(np.float64), tau)
    assert np.array_equal(B.mask_bits_to_bool(ex["mask_bits"], cfg.E), mask)
    got = B.from_device(y, cfg.dtype)
    err, n_allow = _check(oracle, layer, x, mask, got, cfg.dtype)
    # the hidden quantisation is part of what is computed: against the layer that quantises
    # only the input the result is farther off
    xq, _ = oracle.quantize_rows_e4m3(x)
    err_x8 = tokenwise_rel_err(got, oracle_ffn(oracle, layer, xq, mask))
    print(f"  density={mask.mean():.3f} err={err:.3e} (tokens on the one-step allowance: {n_allow}; "
          f"against unquantised hidden rows: {err_x8:.3e})", flush=True)
    assert err_x8 > err
    # explicit lists (Bernoulli decisions), with a token that has no expert
    m2 = wl.bernoulli_mask(T, cfg.E, 0.3, seed=T)
    m2[T // 2] = 0
    offs, lst = lists_from_mask(m2, shuffle_seed=2)
    y2 = B.dmoe_expert_ffn(L, xd, torch.from_numpy(offs).cuda(),
                           torch.from_numpy(np.concatenate([lst, np.zeros(1, np.int32)])).cuda())
    torch.cuda.synchronize()
    _check(oracle, layer, x, m2, B.from_device(y2, cfg.dtype), cfg.dtype)


def test_experts_narrower_than_their_rows_and_plain_experts(B, oracle):
    """48 gated neurons in rows of 64 (the padding neurons are zeros on both sides of the 8-bit
    product) and plain GELU experts of 64 with biases."""
    import torch
    from dataclasses import replace
    for cfg in (replace(small_cfg("cfg4", 333, 12), m=48),
                replace(small_cfg("cfg2", 300, 20), m=64)):
        layer = _a8_layer(cfg, 4)
        x = wl.make_input(cfg, 4)
        mask = wl.bernoulli_mask(cfg.T, cfg.E, 0.4, seed=1)
        offs, lst = lists_from_mask(mask)
        y = B.dmoe_expert_ffn(B.Layer(layer, cfg.dtype), B.to_device(x, cfg.dtype), torch.from_numpy(offs).cuda(),
                              torch.from_numpy(np.concatenate([lst, np.zeros(1, np.int32)])).cuda())
        torch.cuda.synchronize()
        err, n_allow = _check(oracle, layer, x, mask, B.from_device(y, cfg.dtype), cfg.dtype)
        print(f"fully 8-bit m={cfg.m} gated={cfg.gated} err={err:.3e} ({n_allow} tokens on the allowance)", flush=True)


def test_negative_and_zero_weight_scales(B, oracle):
    """The block scales of the 8-bit matrix instruction carry no sign: a negative down scale
    flips the expert's codes at pack time, a zero scale silences the expert."""
    import torch
    cfg = small_cfg("cfg4", 200, 8)
    layer = _a8_layer(cfg, 5)
    layer["w8"] = dict(layer["w8"])
    scales = layer["w8"]["scales"].copy()
    scales[1, 2] = -scales[1, 2]
    scales[2, 2] = 0.0
    layer["w8"]["scales"] = scales
    # the oracle's weights are the dequantised ones: redo them with the bent scales
    layer["w_down"] = np.asarray(layer["w_down"], dtype=np.float64).copy()
    layer["w_down"][1] = -layer["w_down"][1]
    layer["w_down"][2] = 0.0
    x = wl.make_input(cfg, 5)
    mask = np.ones((cfg.T, cfg.E), np.uint8)
    offs, lst = lists_from_mask(mask)
    y = B.dmoe_expert_ffn(B.Layer(layer, cfg.dtype), B.to_device(x, cfg.dtype), torch.from_numpy(offs).cuda(),
                          torch.from_numpy(np.concatenate([lst, np.zeros(1, np.int32)])).cuda())
    torch.cuda.synchronize()
    _check(oracle, layer, x, mask, B.from_device(y, cfg.dtype), cfg.dtype)


def test_static_workspace_graph_replay_and_no_tokens(B):
    import torch
    cfg = small_cfg("cfg4", 200, 16)
    L = B.Layer(_a8_layer(cfg, 9), cfg.dtype)
    tau = float(np.float32(0.3))
    xs = [B.to_device(wl.make_input(cfg, 30 + i), cfg.dtype) for i in range(3)]
    y_ref, _ = B.dmoe_forward(L, xs[0], tau)
    y_static = B.dmoe_forward_static(L, xs[0], tau)
    torch.cuda.synchronize()
    assert torch.equal(y_static, y_ref)
    x_in, y_graph, y_eager = xs[0].clone(), torch.empty_like(xs[0]), torch.empty_like(xs[0])
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.dmoe_forward(L, x_in, tau, y=y_graph)
    for i in range(3):
        x_in.copy_(xs[i])
        y_graph.zero_()
        g.replay()
        B.dmoe_forward(L, xs[i], tau, y=y_eager)
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_eager), f"replay {i}"
    y0, _ = B.dmoe_forward(L, xs[0][:0], tau)
    assert tuple(y0.shape) == (0, cfg.d)
