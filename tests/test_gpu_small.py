"""The small-token (decode) path: T <= 16 tokens, weight-streaming kernels."""
import numpy as np
import pytest

from helpers import TOL, lists_from_mask, oracle_ffn, small_cfg, tokenwise_rel_err
from paper_2310_04361_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2310_04361_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("name,T,E", [("cfg5a", 16, None), ("cfg5a", 5, 64), ("cfg5a", 1, 32),
                                      ("cfg5b", 16, None), ("cfg5b", 3, None), ("cfg2", 16, None),
                                      ("cfg2", 9, None), ("paper", 16, None)])
def test_small_forward_and_expert_ffn(B, oracle, name, T, E):
    import torch
    cfg = small_cfg(name, T, E)
    print(f"small {name} T={T} E={cfg.E}", flush=True)
    layer, x = wl.make_layer(cfg, 4), wl.make_input(cfg, 4)
    L = B.Layer(layer, cfg.dtype)
    xd = B.to_device(x, cfg.dtype)
    for tau in (0.5, 0.0):
        tau32 = float(np.float32(tau))
        y, ex = B.dmoe_forward(L, xd, tau32, want_scores=True, want_mask=True, want_lists=True)
        torch.cuda.synchronize()
        s = ex["scores"].cpu().numpy()
        ref_mask, _ = oracle.select(s.astype(np.float64), tau32)
        assert np.array_equal(B.mask_bits_to_bool(ex["mask_bits"], cfg.E), ref_mask)
        offsets = ex["offsets"].cpu().numpy()
        lists = ex["token_lists"].cpu().numpy()
        for e in range(cfg.E):
            assert lists[offsets[e]:offsets[e + 1]].tolist() == np.flatnonzero(ref_mask[:, e]).tolist()
        ref = oracle_ffn(oracle, layer, x, ref_mask)
        err = tokenwise_rel_err(B.from_device(y, cfg.dtype), ref)
        print(f"  tau={tau} density={ref_mask.mean():.3f} err={err:.3e}", flush=True)
        assert err <= TOL["bf16"]
    # explicit lists, with a token that has no expert and experts nobody selected
    mask = wl.bernoulli_mask(T, cfg.E, 0.3, seed=T + 1)
    mask[T // 2] = 0
    mask[:, :3] = 0
    offs, lst = lists_from_mask(mask, shuffle_seed=1)
    y = B.dmoe_expert_ffn(L, xd, torch.from_numpy(offs).cuda(),
                          torch.from_numpy(np.concatenate([lst, np.zeros(1, np.int32)])).cuda())
    torch.cuda.synchronize()
    got = B.from_device(y, cfg.dtype)
    assert tokenwise_rel_err(got, oracle_ffn(oracle, layer, x, mask)) <= TOL["bf16"]
    b2 = layer["b_down"] if layer["b_down"] is not None else np.zeros(cfg.d)
    assert np.array_equal(got[T // 2], b2)
