"""Layers with 8-bit expert weights AND 8-bit expert inputs (weight format DMOE_W_FP8_E4M3_X8, the
lower-precision layers of Appendix C).  The experts read every token's row quantised to E4M3 with
a power-of-two scale; the oracle quantises the rows itself (oracle.quantize_rows_e4m3) and runs
its fp64 experts on them, so the bar stays the bf16 bar.  Wide experts (128 neurons, 64 if gated)
run the 8-bit matrix-core up-projection above 16 tokens; other shapes and the small-token path
run their bf16 kernels on the quantised rows."""
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


def _x8_layer(cfg, seed):
    layer = wl.quantize_experts_e4m3(wl.make_layer(cfg, seed))
    layer["x8"] = True
    return layer


def test_quantised_rows_bit_exact_through_an_identity_layer(B, oracle):
    """Four ReLU experts of 128 neurons whose up rows are +-unit vectors and whose down rows are
    +-unit vectors: with every expert selected, y_j = relu(xq_j) - relu(-xq_j) = xq_j exactly (one
    term is zero, every value is a bf16 number), so y must equal the oracle's quantised rows
    bit for bit -- including rows with exact ties, subnormal magnitudes and a zero row."""
    import torch
    d, E, m, T = 256, 4, 128, 333
    eye = np.eye(d)
    w_up = np.stack([eye[:128], eye[128:], -eye[:128], -eye[128:]])          # [E, m, d]
    w_down = w_up.copy()
    layer = {"w_up": w_up, "w_gate": None, "b_up": None, "w_down": w_down, "b_down": None,
             "r_w1": np.zeros((32, d)), "r_b1": None, "r_w2": np.zeros((E, 32)), "r_b2": None,
             "act": "relu", "gated": False}
    layer = wl.quantize_experts_e4m3(layer)          # +-1 and 0 are E4M3 numbers: scales 2^-8 .. 1
    layer["x8"] = True
    rng = np.random.default_rng(4)
    x = wl.round_storage(rng.standard_normal((T, d)) * np.exp(rng.normal(0, 3, (T, 1))), "bf16")
    x[7] = 0.0
    # ties: 17, 19, 21 lie half-way between E4M3 neighbours (step 2 between 16 and 32); 448 pins s = 1
    x[11, :6] = [448.0, 17.0, 19.0, -21.0, 2.0 ** -10, 3 * 2.0 ** -10]
    x[11, 6:] = 0.0
    L = B.Layer(layer, "bf16")
    mask = np.ones((T, E), np.uint8)
    offs, lst = lists_from_mask(mask)
    y = B.dmoe_expert_ffn(L, B.to_device(x, "bf16"), torch.from_numpy(offs).cuda(),
                          torch.from_numpy(np.concatenate([lst, np.zeros(1, np.int32)])).cuda())
    torch.cuda.synchronize()
    xq, _ = oracle.quantize_rows_e4m3(x)
    got = B.from_device(y, "bf16")
    assert np.array_equal(got, xq)
    assert got[11, :6].tolist() == [448.0, 16.0, 20.0, -20.0, 0.0, 2.0 ** -8]


@pytest.mark.parametrize("name,T,E", [("cfg4", 300, 16), ("cfg4", 700, 8), ("paper", 260, 8),
                                      ("cfg2", 300, 32), ("gemma_paper", 200, 64),
                                      ("cfg5a", 16, 64), ("cfg5b", 5, None), ("cfg4", 17, 16)])
def test_forward_with_8bit_inputs(B, oracle, name, T, E):
    import torch
    cfg = small_cfg(name, T, E)
    print(f"8-bit inputs {name} T={T} E={cfg.E}", flush=True)
    layer = _x8_layer(cfg, 3)
    x = wl.make_input(cfg, 3)
    L = B.Layer(layer, cfg.dtype)
    tau = float(np.float32(0.4))
    xd = B.to_device(x, cfg.dtype)
    y, ex = B.dmoe_forward(L, xd, tau, want_scores=True, want_mask=True)
    torch.cuda.synchronize()
    s = ex["scores"].cpu().numpy().astype(np.float64)
    mask, _ = oracle.select(s, tau)
    assert np.array_equal(B.mask_bits_to_bool(ex["mask_bits"], cfg.E), mask)
    # the router reads the original rows: same scores as the layer without 8-bit inputs
    plain = {k: v for k, v in layer.items() if k != "x8"}
    _, ex2 = B.dmoe_forward(B.Layer(plain, cfg.dtype), xd, tau, want_scores=True)
    torch.cuda.synchronize()
    assert torch.equal(ex["scores"], ex2["scores"])
    xq, _ = oracle.quantize_rows_e4m3(x)
    ref = oracle_ffn(oracle, layer, xq, mask)
    err = tokenwise_rel_err(B.from_device(y, cfg.dtype), ref)
    # ... and the quantisation is visible: against the unquantised input the result is farther off
    err_plain = tokenwise_rel_err(B.from_device(y, cfg.dtype), oracle_ffn(oracle, layer, x, mask))
    print(f"  density={mask.mean():.3f} err={err:.3e} (against unquantised input: {err_plain:.3e})", flush=True)
    assert err <= TOL[cfg.dtype]
    assert err_plain > err
    # explicit lists (Bernoulli decisions), with a token that has no expert
    m2 = wl.bernoulli_mask(T, cfg.E, 0.3, seed=T)
    m2[T // 2] = 0
    offs, lst = lists_from_mask(m2, shuffle_seed=2)
    y2 = B.dmoe_expert_ffn(L, xd, torch.from_numpy(offs).cuda(),
                           torch.from_numpy(np.concatenate([lst, np.zeros(1, np.int32)])).cuda())
    torch.cuda.synchronize()
    assert tokenwise_rel_err(B.from_device(y2, cfg.dtype), oracle_ffn(oracle, layer, xq, m2)) <= TOL[cfg.dtype]


def _oracle_x8(oracle, layer, x, mask):
    xq, _ = oracle.quantize_rows_e4m3(x)
    return oracle_ffn(oracle, layer, xq, mask)


@pytest.mark.parametrize("name,T,E,k", [("cfg4", 300, 16, 3), ("cfg2", 200, 32, 5), ("cfg5a", 9, 64, 4)])
def test_top_k_gate_with_8bit_inputs(B, oracle, name, T, E, k):
    import torch
    cfg = small_cfg(name, T, E)
    print(f"8-bit inputs, top-{k} gate, {name} T={T}", flush=True)
    layer, x = _x8_layer(cfg, 6), wl.make_input(cfg, 6)
    y, ex = B.dmoe_forward_topk(B.Layer(layer, cfg.dtype), B.to_device(x, cfg.dtype), k,
                                want_scores=True, want_mask=True)
    torch.cuda.synchronize()
    mask = oracle.select_topk(ex["scores"].cpu().numpy().astype(np.float64), k)
    assert np.array_equal(B.mask_bits_to_bool(ex["mask_bits"], cfg.E), mask)
    assert tokenwise_rel_err(B.from_device(y, cfg.dtype), _oracle_x8(oracle, layer, x, mask)) <= TOL[cfg.dtype]


@pytest.mark.parametrize("name,T,E", [("cfg5b", 16, None), ("cfg5b", 40, None), ("cfg4", 100, 16)])
def test_group_of_layers_with_8bit_inputs(B, oracle, name, T, E):
    """Three layers of one shape on one input (Sec. 3.5): the same outputs as three single calls,
    bit for bit, and the oracle's on its own quantised rows."""
    import torch
    cfg = small_cfg(name, T, E)
    print(f"8-bit inputs, group of 3, {name} T={T}", flush=True)
    layers = [_x8_layer(cfg, 20 + i) for i in range(3)]
    Ls = [B.Layer(l, cfg.dtype) for l in layers]
    x = wl.make_input(cfg, 20)
    xd = B.to_device(x, cfg.dtype)
    taus = [float(np.float32(t)) for t in (0.3, 0.5, 0.7)]
    ys = B.dmoe_forward_group(Ls, xd, taus)
    torch.cuda.synchronize()
    for L, layer, tau, y in zip(Ls, layers, taus, ys):
        y1, ex = B.dmoe_forward(L, xd, tau, want_scores=True)
        torch.cuda.synchronize()
        assert torch.equal(y, y1)
        mask, _ = oracle.select(ex["scores"].cpu().numpy().astype(np.float64), tau)
        assert tokenwise_rel_err(B.from_device(y, cfg.dtype), _oracle_x8(oracle, layer, x, mask)) <= TOL[cfg.dtype]


@pytest.mark.parametrize("T", [1, 15, 16, 17, 63, 64, 65, 257])
def test_token_counts_around_the_kernel_switches_with_8bit_inputs(B, oracle, T):
    """16 | 17 tokens is the switch from the small-token kernels to the 8-bit matrix-core
    up-projection; 64 and 256 are its wavefront and work-item sizes."""
    import torch
    cfg = small_cfg("cfg4", T, 16)
    layer, x = _x8_layer(cfg, 8), wl.make_input(cfg, 8)
    tau = float(np.float32(0.3))
    y, ex = B.dmoe_forward(B.Layer(layer, cfg.dtype), B.to_device(x, cfg.dtype), tau, want_scores=True)
    torch.cuda.synchronize()
    mask, _ = oracle.select(ex["scores"].cpu().numpy().astype(np.float64), tau)
    err = tokenwise_rel_err(B.from_device(y, cfg.dtype), _oracle_x8(oracle, layer, x, mask))
    print(f"8-bit inputs T={T} err={err:.3e}", flush=True)
    assert err <= TOL[cfg.dtype]


def test_no_tokens_with_8bit_inputs(B):
    import torch
    cfg = small_cfg("cfg4", 4, 16)
    L = B.Layer(_x8_layer(cfg, 8), cfg.dtype)
    y, _ = B.dmoe_forward(L, B.to_device(wl.make_input(cfg, 8)[:0], cfg.dtype), 0.5)
    torch.cuda.synchronize()
    assert tuple(y.shape) == (0, cfg.d)


def test_static_workspace_and_graph_replay_with_8bit_inputs(B):
    """The row quantiser is one more kernel on the same stream: the static-workspace entry gives
    the same bits as dmoe_forward, and a captured forward replays like the eager one."""
    import torch
    cfg = small_cfg("cfg4", 200, 16)
    L = B.Layer(_x8_layer(cfg, 9), cfg.dtype)
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
