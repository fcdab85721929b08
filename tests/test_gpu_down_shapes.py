"""Every expert size and launch shape of the bf16 down-projection (Sec. 3.2: the sum over the
selected experts) against the oracle on sampled tokens.

The matrix-core merge is compiled per packing of the experts' 8-neuron pieces into MFMA k-steps
(2, 3, 4 or 8 k-steps per stage of one or two experts) and per workgroup shape (256 columns
with one or two workgroups per CU, 384 columns); the benchmark configurations reach only a few
of these, so synthetic layers of every expert size run here at token counts that select each
shape.  Decisions are Bernoulli(p) draws (the device of Sec. 4.4) well above the density at
which the pair-proportional kernel takes over."""
import numpy as np
import pytest

from helpers import TOL, lists_from_mask, oracle_ffn, tokenwise_rel_err
from paper_2310_04361_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2310_04361_amd import binding
    binding.lib()
    return binding


def _cfg(T, d, E, m, gated):
    return wl.Config(f"m{m}", T, d, E, m, 64, gated, "gelu_tanh" if gated else "gelu_erf", "bf16",
                     (0.5,), ffn_bias=not gated)


# one narrow workgroup per CU (few tokens): every k-step packing, plain and gated; expert counts
# from 1 up, not multiples of the 32-expert mask batch or of the 4-stage loop trip, and beyond
# several batches (an expert of exactly 128 neurons is walked as two units of 64: two stages and
# one mask bit per expert)
ONE_PER_CU = [(300, 256, 20, m, False) for m in (8, 16, 24, 32, 40, 48, 64, 72, 96, 100, 128)] + \
             [(300, 256, 37, m, True) for m in (16, 32, 48, 64)] + \
             [(200, 256, 70, 24, False)] + \
             [(200, 256, E, 24, False) for E in (1, 3, 5, 33, 65, 130, 300)] + \
             [(200, 256, E, 64, False) for E in (1, 33, 100)] + \
             [(200, 256, E, 128, False) for E in (1, 3, 17, 33, 70)] + \
             [(128, 256, 2048, 8, False), (96, 512, 4096, 16, True)] + \
             [(300, 256, 37, m, True) for m in (1, 3, 5, 8)] + \
             [(1000, 512, 600, 8, True)]
# (many small experts up to the largest count; gated experts of at most 8 neurons take the
# up-projection kernel that keeps an expert's up and gate rows in one weight tile)
# 384-column workgroups: d = 768 and 10880 < T <= 16384
WIDE = [(11000, 768, 16, m, False) for m in (16, 32, 48, 64, 128)] + [(12000, 768, 12, 32, True)]
# more narrow workgroups than CUs (two per CU up to 4 k-steps per stage, else several rounds)
MANY = [(16500, 512, 12, m, False) for m in (16, 24, 32, 64, 128)]


@pytest.mark.parametrize("T,d,E,m,gated", ONE_PER_CU + WIDE + MANY)
def test_down_projection_shapes(B, oracle, T, d, E, m, gated):
    import torch
    cfg = _cfg(T, d, E, m, gated)
    print(f"down shapes T={T} d={d} E={E} m={m} gated={gated}", flush=True)
    layer, x = wl.make_layer(cfg, 3), wl.make_input(cfg, 3)
    L = B.Layer(layer, cfg.dtype)
    mask = wl.bernoulli_mask(T, E, 0.3, seed=m + T)
    mask[1] = 0          # a token with no expert
    if E > 1:
        mask[:, E - 1] = 0   # an expert with no token
    offsets, lists = lists_from_mask(mask)
    lists_dev = torch.from_numpy(np.concatenate([lists, np.zeros(1, np.int32)])).cuda()
    y = B.dmoe_expert_ffn(L, B.to_device(x, cfg.dtype), torch.from_numpy(offsets).cuda(), lists_dev)
    torch.cuda.synchronize()
    got = B.from_device(y, cfg.dtype)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(7)
    idx = np.unique(np.concatenate([[i for i in (0, 1, 63, 64, 127, 128, T - 1) if i < T],
                                    rng.choice(T, min(96, T), replace=False)]))
    ref = oracle_ffn(oracle, layer, x[idx], mask[idx])
    err = tokenwise_rel_err(got[idx], ref)
    print(f"  err={err:.3e}", flush=True)
    assert err <= TOL[cfg.dtype]
