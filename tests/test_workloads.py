"""Host-side checks of the synthetic-input module and the Appendix B cost model."""
import numpy as np
import torch

from paper_2310_04361_amd import cost_model, workloads as wl


def test_bf16_rounding_matches_torch():
    a = np.random.default_rng(0).standard_normal(10000) * np.exp(np.random.default_rng(1).uniform(-20, 20, 10000))
    bits = wl.f64_to_bf16_bits(a)
    ref = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16)
    assert np.array_equal(bits, ref.view(torch.int16).numpy().view(np.uint16))
    back = wl.bf16_bits_to_f64(bits)
    assert np.array_equal(back, ref.to(torch.float64).numpy())
    assert np.array_equal(wl.round_bf16(back), back)          # idempotent


def test_draws_are_seeded_and_representable():
    cfg = wl.with_tokens(wl.CONFIGS["cfg2"], 8)
    a, b = wl.make_layer(cfg, 3), wl.make_layer(cfg, 3)
    for k in ("w_up", "w_down", "b_up", "b_down", "r_w1", "r_w2"):
        assert np.array_equal(a[k], b[k])
        assert np.array_equal(wl.round_bf16(a[k]), a[k])
    assert a["w_gate"] is None and a["r_b1"] is None
    assert not np.array_equal(wl.make_layer(cfg, 4)["w_up"], a["w_up"])
    g = wl.make_layer(wl.with_tokens(wl.CONFIGS["cfg4"], 8), 0)
    assert g["w_gate"].shape == (256, 64, 2048) and g["b_up"] is None
    x = wl.make_input(wl.with_tokens(wl.CONFIGS["cfg3"], 2000), 0)
    assert x.shape == (2000, 768)
    assert np.std(np.log(np.linalg.norm(x, axis=1))) > 0.8     # log-normal row scales took


def test_config_shapes():
    c = wl.CONFIGS
    assert (c["cfg1"].H, c["cfg2"].H, c["cfg4"].H, c["cfg5b"].H, c["paper"].H) == (256, 3072, 16384, 768, 3072)
    assert c["cfg2"].T == 16384 and c["cfg3"].T == 50432 and c["cfg4"].T == 4096


def test_cost_model_matches_appendix_b():
    # Appendix B: ratio = k/n + d_h (1 + n/d_m) / (2 e d_m); with d_m = 768, e = 4, n = 128,
    # d_h = 128 the router term is 0.0243.
    d, e, n, dh = 768, 4, 128, 128
    m = e * d // n
    router_term = dh * (1 + n / d) / (2 * e * d)
    assert abs(router_term - 0.0243) < 5e-5
    for k in (0, 1, 17, 128):
        assert abs(cost_model.cost_ratio(k, d, n, m, dh) - (k / n + router_term)) < 1e-12
    assert cost_model.dense_ffn_macs(d, e * d) == 2 * e * d * d
    assert cost_model.expert_macs(d, m) * n == cost_model.dense_ffn_macs(d, e * d)
    assert cost_model.executed_flops(10, 2048, 64, gated=True) == 10 * 786432


def test_e4m3_quantiser_is_exact_storage_rounding():
    """Every code decodes (by the format's definition, written out here) to the value the harness
    hands to the oracle; scales are powers of two; the largest weight of a matrix uses the top
    binade; quantising twice changes nothing."""
    cfg = wl.with_tokens(wl.CONFIGS["cfg5b"], 4)
    layer = wl.make_layer(cfg, 5)
    q = wl.quantize_experts_e4m3(layer)
    codes, scales = q["w8"]["w_up"], q["w8"]["scales"]
    assert codes.dtype == np.uint8 and codes.shape == layer["w_up"].shape
    assert np.all(np.exp2(np.round(np.log2(scales))) == scales)
    sign = np.where(codes & 0x80, -1.0, 1.0)
    e, m = ((codes >> 3) & 15).astype(np.int64), (codes & 7).astype(np.float64)
    mag = np.where(e == 0, m * 2.0 ** -9, (8 + m) * np.exp2((e - 10).astype(np.float64)))
    assert not np.any((codes & 0x7f) == 0x7f)                       # no NaN codes
    assert np.array_equal(sign * mag * scales[:, 0][:, None, None], q["w_up"])
    assert (mag.reshape(cfg.E, -1).max(axis=1) >= 256).all()        # top binade of 448 used
    rel = np.abs(q["w_up"] - layer["w_up"]).max() / np.abs(layer["w_up"]).max()
    assert rel <= 2.0 ** -4                                         # 3 mantissa bits
    q2 = wl.quantize_experts_e4m3({k: v for k, v in q.items() if k != "w8"})
    assert np.array_equal(q2["w_up"], q["w_up"]) and np.array_equal(q2["w8"]["w_up"], codes)
