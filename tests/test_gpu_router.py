"""dmoe_router on the GPU against the oracle's router (Sec. 3.3)."""
import numpy as np
import pytest

from helpers import TOL, small_cfg, tokenwise_rel_err
from paper_2310_04361_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2310_04361_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("name,T,E", [
    ("cfg1", 128, None), ("cfg1", 5, None),
    ("cfg2", 300, None), ("cfg2", 16, None), ("cfg2", 1, None),
    ("cfg3", 333, None),            # router biases + log-normal row scales
    ("cfg4", 150, None), ("cfg5b", 16, None), ("paper", 100, None),
])
def test_router_matches_oracle(B, oracle, name, T, E):
    import torch
    cfg = small_cfg(name, T, E)
    print(f"router {name} T={T}", flush=True)
    layer, x = wl.make_layer(cfg, 0), wl.make_input(cfg, 0)
    L = B.Layer(layer, cfg.dtype)
    s = B.dmoe_router(L, B.to_device(x, cfg.dtype))
    torch.cuda.synchronize()
    ref = oracle.router(x, layer["r_w1"], layer["r_b1"], layer["r_w2"], layer["r_b2"])
    got = s.cpu().numpy().astype(np.float64)
    assert (got >= 0).all()
    assert tokenwise_rel_err(got, ref) <= TOL[cfg.dtype]
