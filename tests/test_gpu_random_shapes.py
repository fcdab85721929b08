"""Whole bf16 layers of seeded random shapes against the oracle (Sec. 3.2 - 3.4, Appendix G).

The benchmark configurations and the per-kernel shape tests fix one parameter at a time; here
every case draws all of them together -- token count (small-token path, a ragged few hundred,
over a thousand), width, number and size of experts, router width, gated or plain experts,
biases, threshold or top-k gate, bf16 or 8-bit expert weights -- so that combinations nobody listed by hand are exercised.
The scores of sampled tokens are checked against the oracle's router, the gate bit for bit on
the library's own fp32 scores, the lists against the mask,
and the output of sampled tokens against the oracle's experts on that mask."""
import numpy as np
import pytest

from helpers import TOL, check_fully_8bit, oracle_ffn, tokenwise_rel_err
from paper_2310_04361_amd import workloads as wl

pytestmark = pytest.mark.gpu

N_CASES = 72


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2310_04361_amd import binding
    binding.lib()
    return binding


def draw_case(i):
    rng = np.random.default_rng(1000 + i)
    gated = bool(rng.integers(2))
    T = int((rng.integers(1, 17), rng.integers(17, 400), rng.integers(400, 1600))[i % 3])
    d = int(rng.choice([256, 512, 768, 1024]))
    E = int(rng.integers(1, 240)) if i % 5 else int(rng.integers(400, 1200))
    m = int(rng.integers(1, 65 if gated else 129))
    if i % 4 == 1:
        m = int(rng.integers(1, 17))  # small experts: the packings with several experts per stage
    d_h = int(rng.choice([32, 64, 128, 256]))
    act = "gelu_tanh" if gated else str(rng.choice(["relu", "gelu_erf", "gelu_tanh"]))
    cfg = wl.Config(f"rand{i}", T, d, E, m, d_h, gated, act, "bf16", (0.5,),
                    ffn_bias=(not gated) and bool(rng.integers(2)),
                    router_bias=bool(rng.integers(2)))
    tau = float(np.float32(rng.choice([0.0, 0.2, 0.5, 0.8, 0.95])))
    k = int(rng.integers(1, E + 1)) if i % 7 == 3 else None
    return cfg, tau, k, i % 6 == 2   # every sixth layer stores its expert matrices in E4M3


@pytest.mark.parametrize("i", range(N_CASES))
def test_random_layer_matches_oracle(B, oracle, i):
    import torch
    cfg, tau, k, e4m3 = draw_case(i)
    print(f"random layer {i}: T={cfg.T} d={cfg.d} E={cfg.E} m={cfg.m} d_h={cfg.d_h} "
          f"gated={cfg.gated} act={cfg.act} ffn_bias={cfg.ffn_bias} router_bias={cfg.router_bias} "
          f"tau={tau} k={k} e4m3={e4m3}", flush=True)
    layer, x = wl.make_layer(cfg, i), wl.make_input(cfg, i)
    if e4m3:  # the oracle gets the dequantised weights, which are bf16 numbers
        layer = wl.quantize_experts_e4m3(layer)
    L = B.Layer(layer, cfg.dtype)
    y, ex = B.dmoe_forward(L, B.to_device(x, cfg.dtype), tau, want_scores=True, want_mask=True,
                           want_lists=True, top_k=k)
    torch.cuda.synchronize()
    s = ex["scores"].cpu().numpy()
    assert np.isfinite(s).all() and (s >= 0).all()
    if k is None:
        ref_mask, _ = oracle.select(s.astype(np.float64), tau)
    else:
        ref_mask = oracle.select_topk(s.astype(np.float64), k)
    got_mask = B.mask_bits_to_bool(ex["mask_bits"], cfg.E)
    assert np.array_equal(got_mask, ref_mask)
    offsets = ex["offsets"].cpu().numpy()
    lists = ex["token_lists"].cpu().numpy()
    assert offsets[0] == 0 and offsets[-1] == ref_mask.sum()
    for e in range(cfg.E):
        assert lists[offsets[e]:offsets[e + 1]].tolist() == np.flatnonzero(ref_mask[:, e]).tolist()
    got = B.from_device(y, cfg.dtype)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(i)
    idx = np.unique(np.concatenate([[t for t in (0, 15, 16, 63, 64, 127, 128, cfg.T - 1) if t < cfg.T],
                                    rng.choice(cfg.T, min(48, cfg.T), replace=False)]))
    ref_s = oracle.router(x[idx], layer["r_w1"], layer["r_b1"], layer["r_w2"], layer["r_b2"])
    assert tokenwise_rel_err(s[idx], ref_s) <= TOL[cfg.dtype]
    ref_y = oracle_ffn(oracle, layer, x[idx], ref_mask[idx])
    err = tokenwise_rel_err(got[idx], ref_y)
    print(f"  density={ref_mask.mean():.3f} err={err:.3e}", flush=True)
    assert err <= TOL[cfg.dtype]


@pytest.mark.parametrize("fmt", ["x8", "a8"])
@pytest.mark.parametrize("i", range(0, N_CASES, 3))
def test_random_layer_with_8bit_activations(B, oracle, i, fmt):
    """Every third draw again with 8-bit expert inputs (x8) and with 8-bit hidden activations as
    well (a8): whatever kernels the shape selects, the layer must compute the format's
    definition -- the oracle's experts on the oracle's quantised rows."""
    import torch
    cfg, tau, k, _ = draw_case(i + 1)   # the ragged few-hundred-token draws, mostly
    print(f"random 8-bit layer {i + 1} ({fmt}): T={cfg.T} d={cfg.d} E={cfg.E} m={cfg.m} gated={cfg.gated} "
          f"act={cfg.act} tau={tau} k={k}", flush=True)
    layer = wl.quantize_experts_e4m3(wl.make_layer(cfg, i))
    layer["x8"] = True
    if fmt == "a8":
        layer["a8"] = True
    x = wl.make_input(cfg, i)
    L = B.Layer(layer, cfg.dtype)
    y, ex = B.dmoe_forward(L, B.to_device(x, cfg.dtype), tau, want_scores=True, want_mask=True, top_k=k)
    torch.cuda.synchronize()
    s = ex["scores"].cpu().numpy().astype(np.float64)
    ref_mask = oracle.select(s, tau)[0] if k is None else oracle.select_topk(s, k)
    assert np.array_equal(B.mask_bits_to_bool(ex["mask_bits"], cfg.E), ref_mask)
    got = B.from_device(y, cfg.dtype)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(i)
    idx = np.unique(np.concatenate([[t for t in (0, 15, 16, 63, 64, cfg.T - 1) if t < cfg.T],
                                    rng.choice(cfg.T, min(32, cfg.T), replace=False)]))
    xq, _ = oracle.quantize_rows_e4m3(x[idx])
    ref = oracle_ffn(oracle, layer, xq, ref_mask[idx], quantize_h=(fmt == "a8"))
    if fmt == "a8":
        err, n_allow = check_fully_8bit(oracle, layer, xq, ref_mask[idx], got[idx], ref, TOL[cfg.dtype],
                                        max_share=0.05)
        print(f"  density={ref_mask.mean():.3f} err={err:.3e} tokens on the one-step allowance: {n_allow}", flush=True)
    else:
        err = tokenwise_rel_err(got[idx], ref)
        print(f"  density={ref_mask.mean():.3f} err={err:.3e}", flush=True)
        assert err <= TOL[cfg.dtype]


@pytest.mark.parametrize("T,d,E,m,gated", [(300, 4096, 16, 64, True), (9, 4096, 16, 64, True),
                                           (9, 8192, 8, 24, False), (130, 8192, 8, 24, False)])
def test_wide_models(B, oracle, T, d, E, m, gated):
    """Model widths beyond the benchmark shapes: 4096 (the widest whose 16 x rows the small-token
    kernels keep in LDS) and 8192 (where up to 16 tokens take the general kernels instead)."""
    import torch
    cfg = wl.Config(f"wide{d}", T, d, E, m, 128, gated, "gelu_tanh", "bf16", (0.5,),
                    ffn_bias=not gated, router_bias=True)
    print(f"wide model T={T} d={d} E={E} m={m} gated={gated}", flush=True)
    layer, x = wl.make_layer(cfg, 11), wl.make_input(cfg, 11)
    L = B.Layer(layer, cfg.dtype)
    tau = float(np.float32(0.5))
    y, ex = B.dmoe_forward(L, B.to_device(x, cfg.dtype), tau, want_scores=True, want_mask=True)
    torch.cuda.synchronize()
    s = ex["scores"].cpu().numpy()
    ref_mask, _ = oracle.select(s.astype(np.float64), tau)
    assert np.array_equal(B.mask_bits_to_bool(ex["mask_bits"], cfg.E), ref_mask)
    idx = np.arange(min(T, 40))
    ref_s = oracle.router(x[idx], layer["r_w1"], layer["r_b1"], layer["r_w2"], layer["r_b2"])
    assert tokenwise_rel_err(s[idx], ref_s) <= TOL[cfg.dtype]
    err = tokenwise_rel_err(B.from_device(y, cfg.dtype)[idx], oracle_ffn(oracle, layer, x[idx], ref_mask[idx]))
    print(f"  err={err:.3e}", flush=True)
    assert err <= TOL[cfg.dtype]


@pytest.mark.parametrize("T,d,E,m,d_h,gated,act,tau", [
    (50, 96, 7, 5, 16, False, "relu", 0.5), (33, 256, 20, 33, 64, True, "gelu_tanh", 0.3),
    (200, 64, 130, 3, 32, False, "gelu_erf", 0.7), (17, 1000, 4, 200, 100, False, "relu", 0.0),
    (1, 40, 3, 9, 8, True, "gelu_tanh", 0.9),
])
def test_fp32_layers_of_other_shapes(B, oracle, T, d, E, m, d_h, gated, act, tau):
    """The fp32 kernels (the exactness configuration) away from the 64-wide benchmark layer: both
    sides compute their own scores, so tokens with a score within 1e-6 of the threshold are left
    out of the comparison (at most a tenth of them)."""
    import torch
    cfg = wl.Config("f32", T, d, E, m, d_h, gated, act, "f32", (tau,), ffn_bias=not gated,
                    router_bias=True)
    print(f"fp32 layer T={T} d={d} E={E} m={m} d_h={d_h} gated={gated} {act} tau={tau}", flush=True)
    layer, x = wl.make_layer(cfg, 21), wl.make_input(cfg, 21)
    L = B.Layer(layer, cfg.dtype)
    tau32 = float(np.float32(tau))
    y, ex = B.dmoe_forward(L, B.to_device(x, cfg.dtype), tau32, want_scores=True, want_mask=True)
    torch.cuda.synchronize()
    ref_y, ref_s, ref_mask = oracle.forward(layer, x, tau32)
    mx = ref_s.max(axis=1, keepdims=True)
    near = (np.abs(ref_s - tau32 * mx) <= 1e-6 * np.maximum(1.0, mx)).any(axis=1) if tau > 0 else np.zeros(T, bool)
    keep = ~near
    assert keep.sum() >= T * 0.9
    assert tokenwise_rel_err(ex["scores"].cpu().numpy(), ref_s) <= 1e-5
    assert np.array_equal(B.mask_bits_to_bool(ex["mask_bits"], E)[keep], ref_mask[keep])
    assert tokenwise_rel_err(B.from_device(y, cfg.dtype)[keep], ref_y[keep]) <= 1e-5
