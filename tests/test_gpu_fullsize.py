"""Full-size runs (the shapes and launch configuration that bench.py times): EVERY token of the
benchmark configurations is compared with the oracle, the large ragged shapes on sampled tokens
of every 128-token chunk, plus properties that hold at any size."""
import numpy as np
import pytest

from helpers import (TOL, check_fully_8bit, elementwise_rel_err, lists_from_mask, oracle_ffn,
                     tokenwise_rel_err, tokenwise_rel_errs)
from paper_2310_04361_amd import workloads as wl

pytestmark = pytest.mark.gpu


_made = {}


def _layer_and_input(cfg, seed):
    """Layer and input of a configuration; the last one drawn is kept (drawing and rounding the
    200 MB of the Gemma-shaped layer takes a minute, and consecutive cases share it)."""
    key = (cfg, seed)
    if key not in _made:
        _made.clear()
        _made[key] = (wl.make_layer(cfg, seed), wl.make_input(cfg, seed))
    return _made[key]


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2310_04361_amd import binding
    binding.lib()
    return binding


# n_sample = 0: every token goes to the oracle
@pytest.mark.parametrize("name,tau,n_sample", [("cfg2", 0.5, 0), ("cfg2", 0.9, 0),
                                               ("cfg3", 0.5, 0), ("cfg4", 0.3, 0),
                                               ("cfg4", 0.6, 0),
                                               # ragged last chunk in the token range where the
                                               # down-projection takes its 384-column shape
                                               ("cfg2:11000", 0.3, 128),
                                               # ragged last group with whole-group router workgroups
                                               ("cfg2:12345", 0.5, 96),
                                               # the paper's own split of its language model: 2048
                                               # experts of 8 neurons, router width 512 (prefill
                                               # and small-token path)
                                               ("gemma_paper:600", 0.5, 32),
                                               # ... and of its text classifier: 512 experts of 6
                                               ("bert_paper:700", 0.5, 48),
                                               ("gemma_paper:12", 0.5, 12),
                                               # both at the sizes bench.py times (windows of the
                                               # up-projection, part-filled work items, several
                                               # items per wavefront)
                                               ("gemma_paper", 0.5, 64), ("bert_paper", 0.5, 96)])
def test_full_size_sampled(B, oracle, name, tau, n_sample):
    import torch
    cfg = wl.CONFIGS[name.split(":")[0]]
    if ":" in name:
        cfg = wl.with_tokens(cfg, int(name.split(":")[1]))
    print(f"full size {name} T={cfg.T} tau={tau}", flush=True)
    layer, x = _layer_and_input(cfg, 0)
    L = B.Layer(layer, cfg.dtype)
    tau32 = float(np.float32(tau))
    y, ex = B.dmoe_forward(L, B.to_device(x, cfg.dtype), tau32, want_scores=True, want_mask=True,
                           want_lists=True)
    torch.cuda.synchronize()
    s = ex["scores"].cpu().numpy()
    mask = B.mask_bits_to_bool(ex["mask_bits"], cfg.E)
    offsets = ex["offsets"].cpu().numpy()
    lists = ex["token_lists"].cpu().numpy()[: offsets[-1]]
    yh = B.from_device(y, cfg.dtype)

    # ---- properties at full size
    assert (mask.sum(axis=1) >= 1).all()                               # the argmax expert is kept
    assert mask[np.arange(cfg.T), s.argmax(axis=1)].all()
    assert offsets[0] == 0 and offsets[-1] == mask.sum()
    assert np.array_equal(np.diff(offsets), mask.sum(axis=0))
    expert_of = np.repeat(np.arange(cfg.E), np.diff(offsets))
    seen = np.zeros_like(mask)
    seen[lists, expert_of] = 1
    assert np.array_equal(seen, mask)                                  # lists == mask, as sets
    starts = np.zeros(len(lists), bool)
    starts[offsets[:-1][np.diff(offsets) > 0]] = True
    assert ((np.diff(lists) > 0) | starts[1:]).all()                   # ascending inside a list
    assert np.isfinite(yh).all()

    # ---- sampled tokens against the oracle
    rng = np.random.default_rng(5)
    if n_sample == 0:
        idx = np.arange(cfg.T)
    else:
        idx = np.unique(np.concatenate([[i for i in (0, 63, 64, cfg.T - 1) if i < cfg.T],
                                        rng.choice(cfg.T, min(n_sample, cfg.T), replace=False)]))
    ref_mask, _ = oracle.select(s[idx].astype(np.float64), tau32)
    assert np.array_equal(mask[idx], ref_mask)                         # bit-exact on the GPU's scores
    ref_s = oracle.router(x[idx], layer["r_w1"], layer["r_b1"], layer["r_w2"], layer["r_b2"])
    assert tokenwise_rel_err(s[idx], ref_s) <= TOL[cfg.dtype]
    ref_y = oracle_ffn(oracle, layer, x[idx], ref_mask)
    err = tokenwise_rel_err(yh[idx], ref_y)
    print(f"  density={mask.mean():.4f} tokens compared={len(idx)} of {cfg.T} err={err:.3e} "
          f"element-wise err={elementwise_rel_err(yh[idx], ref_y):.3e}", flush=True)
    assert err <= TOL[cfg.dtype]

    # ---- run-to-run reproducibility (the merge order is fixed)
    y2, _ = B.dmoe_forward(L, B.to_device(x, cfg.dtype), tau32)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)


def test_full_size_8bit_inputs_every_token(B, oracle):
    """The Gemma-shaped prefill layer at full size with 8-bit expert weights and 8-bit expert
    inputs (the fp8 matrix-core up-projection): every token against the oracle's experts on the
    oracle's quantised rows."""
    import torch
    cfg = wl.CONFIGS["cfg4"]
    print(f"full size cfg4 T={cfg.T} tau=0.3, 8-bit weights and inputs", flush=True)
    base, x = _layer_and_input(cfg, 0)
    layer = wl.quantize_experts_e4m3(base)
    layer["x8"] = True
    L = B.Layer(layer, cfg.dtype)
    tau32 = float(np.float32(0.3))
    y, ex = B.dmoe_forward(L, B.to_device(x, cfg.dtype), tau32, want_scores=True, want_mask=True)
    torch.cuda.synchronize()
    s = ex["scores"].cpu().numpy().astype(np.float64)
    mask, _ = oracle.select(s, tau32)
    assert np.array_equal(B.mask_bits_to_bool(ex["mask_bits"], cfg.E), mask)
    xq, _ = oracle.quantize_rows_e4m3(x)
    ref = oracle_ffn(oracle, layer, xq, mask)
    yh = B.from_device(y, cfg.dtype)
    err = tokenwise_rel_err(yh, ref)
    print(f"  density={mask.mean():.4f} tokens compared={cfg.T} err={err:.3e} "
          f"element-wise err={elementwise_rel_err(yh, ref):.3e}", flush=True)
    assert err <= TOL[cfg.dtype]


@pytest.mark.parametrize("tau", [0.3, 0.6])
def test_full_size_fully_8bit_every_token(B, oracle, tau):
    """The same layer at full size with 8-bit hidden activations as well (both expert products
    on the fp8 matrix cores): every token against the oracle's experts on the oracle's quantised
    input rows, with every selected hidden row quantised by the oracle."""
    import torch
    cfg = wl.CONFIGS["cfg4"]
    print(f"full size cfg4 T={cfg.T} tau={tau}, fully 8-bit", flush=True)
    base, x = _layer_and_input(cfg, 0)
    layer = wl.quantize_experts_e4m3(base)
    layer["x8"] = True
    layer["a8"] = True
    L = B.Layer(layer, cfg.dtype)
    tau32 = float(np.float32(tau))
    y, ex = B.dmoe_forward(L, B.to_device(x, cfg.dtype), tau32, want_scores=True, want_mask=True)
    torch.cuda.synchronize()
    s = ex["scores"].cpu().numpy().astype(np.float64)
    mask, _ = oracle.select(s, tau32)
    assert np.array_equal(B.mask_bits_to_bool(ex["mask_bits"], cfg.E), mask)
    xq, _ = oracle.quantize_rows_e4m3(x)
    ref = oracle_ffn(oracle, layer, xq, mask, quantize_h=True)
    yh = B.from_device(y, cfg.dtype)
    err, n_allow = check_fully_8bit(oracle, layer, xq, mask, yh, ref, TOL[cfg.dtype])
    errs = tokenwise_rel_errs(yh, ref)
    print(f"  density={mask.mean():.4f} tokens compared={cfg.T} err={err:.3e} median={np.median(errs):.3e} "
          f"tokens on the one-step allowance: {n_allow}", flush=True)


def test_paper_shape_full_size_bernoulli(B, oracle):
    """The shape of the latency experiment of Sec. 4.4 (24 experts of 128 neurons, d = 768,
    256 x 197 tokens) under Bernoulli(0.5) decisions through dmoe_expert_ffn: four tokens of
    every 128-token chunk (first, last, two random) against the oracle."""
    import torch
    cfg = wl.CONFIGS["paper"]
    print(f"paper shape T={cfg.T} E={cfg.E} m={cfg.m} Bernoulli(0.5)", flush=True)
    layer, x = wl.make_layer(cfg, 0), wl.make_input(cfg, 0)
    L = B.Layer(layer, cfg.dtype)
    mask = wl.bernoulli_mask(cfg.T, cfg.E, 0.5, seed=3)
    mask[777] = 0                                                     # a token with no expert
    offs, lst = lists_from_mask(mask)
    y = B.dmoe_expert_ffn(L, B.to_device(x, cfg.dtype), torch.from_numpy(offs).cuda(),
                          torch.from_numpy(np.concatenate([lst, np.zeros(1, np.int32)])).cuda())
    torch.cuda.synchronize()
    yh = B.from_device(y, cfg.dtype)
    assert np.isfinite(yh).all()
    rng = np.random.default_rng(9)
    starts = np.arange(0, cfg.T, 128)
    idx = np.unique(np.concatenate([starts, np.minimum(starts + 127, cfg.T - 1),
                                    np.minimum(starts + rng.integers(1, 127, len(starts)), cfg.T - 1),
                                    np.minimum(starts + rng.integers(1, 127, len(starts)), cfg.T - 1),
                                    [777]]))
    ref = oracle_ffn(oracle, layer, x[idx], mask[idx])
    err = tokenwise_rel_err(yh[idx], ref)
    print(f"  pairs={offs[-1]} tokens compared={len(idx)} err={err:.3e} "
          f"element-wise err={elementwise_rel_err(yh[idx], ref):.3e}", flush=True)
    assert err <= TOL[cfg.dtype]
    assert np.array_equal(yh[777], layer["b_down"])


@pytest.mark.parametrize("fmt", ["x8", "a8"])
def test_paper_shape_full_size_bernoulli_8bit(B, oracle, fmt):
    """The same shape and decisions with 8-bit expert inputs (x8) and with 8-bit hidden
    activations as well (a8): plain experts of 128 neurons, several work items per workgroup of
    the 8-bit up-projection, two 64-neuron units per expert in the 8-bit down-projection.  Four
    tokens of every 128-token chunk against the oracle's experts on the oracle's quantised rows."""
    import torch
    cfg = wl.CONFIGS["paper"]
    print(f"paper shape T={cfg.T} E={cfg.E} m={cfg.m} Bernoulli(0.5), {fmt}", flush=True)
    layer = wl.quantize_experts_e4m3(wl.make_layer(cfg, 0))
    layer["x8"] = True
    if fmt == "a8":
        layer["a8"] = True
    x = wl.make_input(cfg, 0)
    L = B.Layer(layer, cfg.dtype)
    mask = wl.bernoulli_mask(cfg.T, cfg.E, 0.5, seed=3)
    mask[777] = 0                                                     # a token with no expert
    offs, lst = lists_from_mask(mask)
    y = B.dmoe_expert_ffn(L, B.to_device(x, cfg.dtype), torch.from_numpy(offs).cuda(),
                          torch.from_numpy(np.concatenate([lst, np.zeros(1, np.int32)])).cuda())
    torch.cuda.synchronize()
    yh = B.from_device(y, cfg.dtype)
    assert np.isfinite(yh).all()
    rng = np.random.default_rng(9)
    starts = np.arange(0, cfg.T, 128)
    idx = np.unique(np.concatenate([starts, np.minimum(starts + 127, cfg.T - 1),
                                    np.minimum(starts + rng.integers(1, 127, len(starts)), cfg.T - 1),
                                    np.minimum(starts + rng.integers(1, 127, len(starts)), cfg.T - 1),
                                    [777]]))
    xq, _ = oracle.quantize_rows_e4m3(x[idx])
    ref = oracle_ffn(oracle, layer, xq, mask[idx], quantize_h=(fmt == "a8"))
    if fmt == "a8":
        err, n_allow = check_fully_8bit(oracle, layer, xq, mask[idx], yh[idx], ref, TOL[cfg.dtype])
        print(f"  pairs={offs[-1]} tokens compared={len(idx)} err={err:.3e} "
              f"tokens on the one-step allowance: {n_allow}", flush=True)
    else:
        err = tokenwise_rel_err(yh[idx], ref)
        print(f"  pairs={offs[-1]} tokens compared={len(idx)} err={err:.3e}", flush=True)
        assert err <= TOL[cfg.dtype]
    assert np.array_equal(yh[777], layer["b_down"])


def test_sizes_beyond_32bit_offsets_take_the_pair_kernel(B, oracle):
    """The matrix-core merge addresses H through 32-bit buffer offsets (below 2 GiB); a layer
    whose worst-case H is larger -- 8200 tokens x 4096 experts of 32-neuron rows -- must go to the
    pair-proportional kernel at any density, and give the same sums (Sec. 3.2)."""
    import torch
    cfg = wl.Config("big_h", 8200, 256, 4096, 8, 64, False, "relu", "bf16", (0.5,), ffn_bias=True)
    print(f"beyond 32-bit offsets: T={cfg.T} E={cfg.E}", flush=True)
    layer, x = wl.make_layer(cfg, 5), wl.make_input(cfg, 5)
    L = B.Layer(layer, cfg.dtype)
    mask = wl.bernoulli_mask(cfg.T, cfg.E, 0.01, seed=5)
    mask[3] = 0
    cols = [np.flatnonzero(mask[:, e]).astype(np.int32) for e in range(cfg.E)]
    offsets = np.concatenate([[0], np.cumsum([len(c) for c in cols])]).astype(np.int32)
    lists = np.concatenate(cols + [np.zeros(1, np.int32)])
    xd = B.to_device(x, cfg.dtype)
    od, ld = torch.from_numpy(offsets).cuda(), torch.from_numpy(lists).cuda()
    B.timing(True)
    y = B.dmoe_expert_ffn(L, xd, od, ld)
    torch.cuda.synchronize()
    t = B.timing_read()
    B.timing(False)
    assert t["expert_down_sparse"][0] == 1 and t["expert_down"][0] == 0
    got = B.from_device(y, cfg.dtype)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(5)
    idx = np.unique(np.concatenate([[0, 3, 127, 128, cfg.T - 1], rng.choice(cfg.T, 60, replace=False)]))
    ref = oracle_ffn(oracle, layer, x[idx], mask[idx])
    err = tokenwise_rel_err(got[idx], ref)
    print(f"  pairs={offsets[-1]} err={err:.3e}", flush=True)
    assert err <= TOL[cfg.dtype]
