"""Layers whose expert matrices are stored in 8-bit floating point (OCP E4M3 with a power-of-two
scale per expert and matrix; the lower-precision experts of Appendix C).  The oracle gets the
dequantised weights -- exactly the numbers the library computes with -- so the bar is the bf16
bar.  Up to 16 tokens the kernels stream the bytes and convert them in registers; above that the
prefill kernels run on bf16 copies made at packing time."""
import numpy as np
import pytest

from helpers import TOL, oracle_ffn, small_cfg, tokenwise_rel_err
from paper_2310_04361_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2310_04361_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("name,T,E", [("cfg5b", 16, None), ("cfg5b", 3, None), ("cfg5a", 16, 64),
                                      ("cfg2", 300, 32), ("cfg4", 200, 16), ("paper", 150, None),
                                      ("gemma_paper", 200, 64), ("gemma_paper", 9, 64)])
def test_forward_with_e4m3_weights(B, oracle, name, T, E):
    import torch
    cfg = small_cfg(name, T, E)
    print(f"e4m3 weights {name} T={T} E={cfg.E}", flush=True)
    layer = wl.quantize_experts_e4m3(wl.make_layer(cfg, 2))
    x = wl.make_input(cfg, 2)
    # every dequantised weight is a bf16 number (the oracle and the library see the same values)
    for k in ("w_up", "w_gate", "w_down"):
        if layer.get(k) is not None:
            assert np.array_equal(wl.round_storage(layer[k], "bf16"), layer[k]), k
    L = B.Layer(layer, cfg.dtype)
    tau = float(np.float32(0.4))
    y, ex = B.dmoe_forward(L, B.to_device(x, cfg.dtype), tau, want_scores=True, want_mask=True)
    torch.cuda.synchronize()
    s = ex["scores"].cpu().numpy().astype(np.float64)
    mask, _ = oracle.select(s, tau)
    assert np.array_equal(B.mask_bits_to_bool(ex["mask_bits"], cfg.E), mask)
    ref = oracle_ffn(oracle, layer, x, mask)
    err = tokenwise_rel_err(B.from_device(y, cfg.dtype), ref)
    print(f"  density={mask.mean():.3f} err={err:.3e}", flush=True)
    assert err <= TOL[cfg.dtype]
    # the same weights handed over as bf16 give the same bits: the 8-bit path changes the
    # storage, not the arithmetic
    plain = {k: v for k, v in layer.items() if k != "w8"}
    y2, _ = B.dmoe_forward(B.Layer(plain, cfg.dtype), B.to_device(x, cfg.dtype), tau)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)


@pytest.mark.parametrize("T", [12, 200])
def test_scales_that_are_not_powers_of_two_are_snapped_on_every_path(B, oracle, T):
    """The header asks for power-of-two scales; a scale that is not one is replaced by the nearest
    power of two at packing time, and the small-token kernels (T <= 16) and the prefill kernels
    use the same snapped copy: both must equal the layer with the snapped scales."""
    import torch
    cfg = small_cfg("cfg5b", T)
    print(f"e4m3 scales off powers of two, T={T}", flush=True)
    layer = wl.quantize_experts_e4m3(wl.make_layer(cfg, 6))
    x = wl.make_input(cfg, 6)
    snapped = dict(layer)                      # the reference layer: scales as powers of two
    bent = dict(layer)
    bent["w8"] = dict(layer["w8"])
    # 1.3 s and 0.8 s both lie closer (in log2) to s than to 2 s or s / 2
    factor = np.where(np.arange(cfg.E)[:, None] % 2 == 0, 1.3, 0.8).astype(np.float32)
    bent["w8"]["scales"] = layer["w8"]["scales"] * factor
    tau = float(np.float32(0.4))
    xd = B.to_device(x, cfg.dtype)
    y_bent, _ = B.dmoe_forward(B.Layer(bent, cfg.dtype), xd, tau)
    y_ref, ex = B.dmoe_forward(B.Layer(snapped, cfg.dtype), xd, tau, want_scores=True)
    torch.cuda.synchronize()
    assert torch.equal(y_bent, y_ref)
    mask, _ = oracle.select(ex["scores"].cpu().numpy().astype(np.float64), tau)
    assert tokenwise_rel_err(B.from_device(y_bent, cfg.dtype), oracle_ffn(oracle, snapped, x, mask)) <= TOL["bf16"]
