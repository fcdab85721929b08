"""dmoe_forward_static -- the entry point for callers that cannot allocate (graph capture,
serving loops): its workspace is a static per-GPU array inside the library.  It must give exactly
what dmoe_forward gives, also on a second call with a smaller input (the array keeps the first
call's contents), and refuse sizes beyond the array before launching anything."""
import ctypes

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


# (configuration, experts, first token count, second -- smaller -- token count)
@pytest.mark.parametrize("name,E,T1,T2", [("cfg2", None, 700, 200),      # prefill kernels
                                          ("cfg5a", 64, 16, 5),          # small-token kernels
                                          ("cfg2", None, 100, 16),       # prefill, then small-token
                                          ("cfg1", None, 128, 31)])      # fp32 kernels
def test_static_workspace_forward_equals_dmoe_forward(B, oracle, name, E, T1, T2):
    import torch
    cfg = small_cfg(name, T1, E)
    print(f"static workspace {name} E={cfg.E} T={T1} then {T2}", flush=True)
    layer, x = wl.make_layer(cfg, 11), wl.make_input(cfg, 11)
    L = B.Layer(layer, cfg.dtype)
    tau32 = float(np.float32(0.5))
    for T in (T1, T2):
        xd = B.to_device(x[:T], cfg.dtype)
        y_ref, ex = B.dmoe_forward(L, xd, tau32, want_scores=True)
        y = B.dmoe_forward_static(L, xd, tau32)
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref), f"T={T}"
        # ... and against the oracle, on the GPU's scores (bf16) / its own (fp32)
        s = ex["scores"].cpu().numpy().astype(np.float64)
        mask, _ = oracle.select(s, tau32)
        if cfg.dtype == "f32":
            ref_s = oracle.router(x[:T], layer["r_w1"], layer["r_b1"], layer["r_w2"], layer["r_b2"])
            m2, _ = oracle.select(ref_s, tau32)
            near = (np.abs(ref_s - tau32 * ref_s.max(axis=1, keepdims=True))
                    <= 1e-6 * np.maximum(1.0, ref_s.max(axis=1, keepdims=True))).any(axis=1)
            keep = ~near & (mask == m2).all(axis=1)
        else:
            keep = np.ones(T, bool)
        ref = oracle_ffn(oracle, layer, x[:T], mask)
        err = tokenwise_rel_err(B.from_device(y, cfg.dtype)[keep], ref[keep])
        print(f"  T={T} err vs oracle {err:.3e}", flush=True)
        assert err <= TOL[cfg.dtype]


def test_static_workspace_refuses_what_does_not_fit(B):
    import torch
    cfg = small_cfg("cfg2", 64)
    layer = wl.make_layer(cfg, 1)
    L = B.Layer(layer, cfg.dtype)
    T = 16384          # worst-case workspace of this layer at 16384 tokens: > 100 MiB
    x = torch.zeros((T, cfg.d), dtype=torch.bfloat16, device="cuda")
    y = torch.full((T, cfg.d), 7.0, dtype=torch.bfloat16, device="cuda")
    rc = B.lib().dmoe_forward_static(L.ref(), x.data_ptr(), T, ctypes.c_float(0.5), y.data_ptr(), None)
    torch.cuda.synchronize()
    assert rc == B.DMOE_ERR_WORKSPACE
    assert b"static" in B.lib().dmoe_last_error()
    assert bool((y == 7.0).all())          # nothing was launched
