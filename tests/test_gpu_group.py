"""dmoe_forward_group: several converted layers of one shape on one input (the attention
projections of Sec. 3.5).  Up to 16 tokens the whole group runs with one launch per stage; its
results must be those of dmoe_forward layer by layer, bit for bit, and inside the tolerance of
the oracle (which gates the GPU's own fp32 scores, as in the other end-to-end tests)."""
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


# "cfg5b/16": the same module at the width that keeps the cost of the projection it replaces
# (16 experts of 24 neurons, hidden width d/2; Sec. 3.5)
@pytest.mark.parametrize("name,T,n_layers", [("cfg5b", 16, 3), ("cfg5b", 5, 4), ("cfg5b", 1, 1),
                                             ("cfg5a", 16, 2), ("cfg5b", 100, 3),
                                             ("cfg5b/16", 16, 3), ("cfg5b/16", 300, 3),
                                             # more experts than the fused small-token gate takes,
                                             # and a count that is no multiple of 4
                                             ("cfg5b/1100", 12, 2), ("cfg5b/30", 16, 3),
                                             # between the fused prefill gate (512) and the
                                             # fused small-token gate (1024)
                                             ("cfg5b/600", 16, 2)])
def test_group_matches_single_layers_and_oracle(B, oracle, name, T, n_layers):
    import torch
    from dataclasses import replace
    cfg = small_cfg(name.split("/")[0], T)
    if "/" in name:
        cfg = replace(cfg, E=int(name.split("/")[1]))
    if name == "cfg5a":
        cfg = replace(cfg, E=64)   # the gated layer with fewer experts keeps the oracle quick
    print(f"group {name} T={T} layers={n_layers}", flush=True)
    x = wl.make_input(cfg, 0)
    layers_np = [wl.make_layer(cfg, 10 + i) for i in range(n_layers)]
    Ls = [B.Layer(l, cfg.dtype) for l in layers_np]
    taus = [float(np.float32(t)) for t in (0.5, 0.3, 0.7, 0.0)[:n_layers]]
    xd = B.to_device(x, cfg.dtype)
    ys = B.dmoe_forward_group(Ls, xd, taus)
    torch.cuda.synchronize()
    for i in range(n_layers):
        y1, ex = B.dmoe_forward(Ls[i], xd, taus[i], want_scores=True, want_mask=True)
        torch.cuda.synchronize()
        assert torch.equal(ys[i], y1), f"layer {i} differs from dmoe_forward"
        s = ex["scores"].cpu().numpy().astype(np.float64)
        mask, _ = oracle.select(s, taus[i])
        assert np.array_equal(B.mask_bits_to_bool(ex["mask_bits"], cfg.E), mask)
        ref = oracle_ffn(oracle, layers_np[i], x, mask)
        err = tokenwise_rel_err(B.from_device(ys[i], cfg.dtype), ref)
        print(f"  layer {i}: tau={taus[i]} density={mask.mean():.3f} err={err:.3e}", flush=True)
        assert err <= TOL[cfg.dtype]
    # a second call on the same buffers gives the same bits (nothing is left over in the workspace)
    ys2 = B.dmoe_forward_group(Ls, xd, taus)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(ys, ys2))
