"""Pins for the oracle's expert execution and merge (Sec. 3.2, Appendix G)."""
import numpy as np
import pytest
import scipy.stats
import torch

from paper_2310_04361_amd import workloads as wl


def _small_layer(rng, T=9, d=7, E=5, m=3, gated=False, bias=True):
    p = dict(
        x=rng.standard_normal((T, d)),
        w_up=rng.standard_normal((E, m, d)),
        w_gate=rng.standard_normal((E, m, d)) if gated else None,
        b_up=rng.standard_normal((E, m)) if (bias and not gated) else None,
        w_down=rng.standard_normal((E, m, d)),
        b_down=rng.standard_normal(d) if bias else None,
    )
    return p


def _ffn(oracle, p, mask, act, gated=False):
    return oracle.expert_ffn(p["x"], p["w_up"], p["w_gate"], p["b_up"], p["w_down"], p["b_down"],
                             mask, act, gated=gated)


def _act_curve(oracle, act, v):
    """A(v) through the oracle: one expert, one neuron, d = 1, unit weights."""
    v = np.asarray(v, dtype=np.float64).reshape(-1, 1)
    one = np.ones((1, 1, 1))
    return oracle.expert_ffn(v, one, None, None, one, None, np.ones((len(v), 1), np.uint8),
                             act)[:, 0]


def test_hand_worked_example(oracle):
    # d = 2, two experts of one neuron, ReLU.
    # x = (1, 2): neuron0 pre = 1*1 + 1*2 - 1 = 2 -> 2 ; neuron1 pre = -1*1 + 0*2 + 0.5 = -0.5 -> 0
    # y = b2 + 2 * (3, -1) + 0 * (10, 10) = (0.5 + 6, -0.5 - 2) = (6.5, -2.5)
    x = [[1.0, 2.0]]
    w_up = [[[1.0, 1.0]], [[-1.0, 0.0]]]
    b_up = [[-1.0], [0.5]]
    w_down = [[[3.0, -1.0]], [[10.0, 10.0]]]
    b_down = [0.5, -0.5]
    both = oracle.expert_ffn(x, w_up, None, b_up, w_down, b_down, [[1, 1]], "relu")
    assert both.tolist() == [[6.5, -2.5]]
    only1 = oracle.expert_ffn(x, w_up, None, b_up, w_down, b_down, [[0, 1]], "relu")
    assert only1.tolist() == [[0.5, -0.5]]          # dead ReLU expert adds exactly nothing
    none = oracle.expert_ffn(x, w_up, None, b_up, w_down, b_down, [[0, 0]], "relu")
    assert none.tolist() == [[0.5, -0.5]]           # no expert: the output is b2
    # x = (-3, 1): neuron1 pre = 3 + 0.5 = 3.5 -> y = b2 + 3.5*(10,10) ; neuron0 pre = -3 -> 0
    y = oracle.expert_ffn([[-3.0, 1.0]], w_up, None, b_up, w_down, b_down, [[1, 1]], "relu")
    assert y.tolist() == [[35.5, 34.5]]


@pytest.mark.parametrize("act", ["relu", "gelu_erf", "gelu_tanh"])
def test_all_experts_equal_dense_ffn(oracle, act):
    """The experts partition the neurons of a dense FFN (Sec. 3.2), so the full mask must give
    the dense layer computed by library matrix products on the un-split matrices."""
    rng = np.random.default_rng(1)
    p = _small_layer(rng, T=17, d=11, E=6, m=4)
    E, m, d = p["w_up"].shape
    W1, b1, W2 = p["w_up"].reshape(E * m, d), p["b_up"].reshape(E * m), p["w_down"].reshape(E * m, d)
    pre = torch.from_numpy(p["x"] @ W1.T + b1)
    if act == "relu":
        a = torch.relu(pre)
    else:
        a = torch.nn.functional.gelu(pre, approximate="tanh" if act == "gelu_tanh" else "none")
    dense = a.numpy() @ W2 + p["b_down"]
    got = _ffn(oracle, p, np.ones((17, E), np.uint8), act)
    np.testing.assert_allclose(got, dense, rtol=0, atol=1e-12)


def test_gated_all_experts_equal_dense_glu(oracle):
    rng = np.random.default_rng(2)
    p = _small_layer(rng, T=13, d=10, E=4, m=5, gated=True, bias=False)
    E, m, d = p["w_up"].shape
    Wg, Wu, Wd = (p[k].reshape(E * m, d) for k in ("w_gate", "w_up", "w_down"))
    g = torch.nn.functional.gelu(torch.from_numpy(p["x"] @ Wg.T), approximate="tanh").numpy()
    dense = (g * (p["x"] @ Wu.T)) @ Wd
    got = _ffn(oracle, p, np.ones((13, E), np.uint8), "gelu_tanh", gated=True)
    np.testing.assert_allclose(got, dense, rtol=0, atol=1e-12)
    # swapping the roles of the gate and up branches must change the result
    q = dict(p, w_gate=p["w_up"], w_up=p["w_gate"])
    assert np.abs(_ffn(oracle, q, np.ones((13, E), np.uint8), "gelu_tanh", gated=True) - dense).max() > 1e-3


def test_gated_with_unit_up_branch_reduces_to_plain(oracle):
    """Append a constant-1 input feature and let the up branch read only it: the gated expert
    becomes A(W_gate x) * 1, i.e. the plain expert with W_up := W_gate and no bias."""
    rng = np.random.default_rng(3)
    T, d, E, m = 8, 6, 3, 4
    x = np.concatenate([rng.standard_normal((T, d)), np.ones((T, 1))], axis=1)
    w_gate = rng.standard_normal((E, m, d + 1))
    w_gate[:, :, d] = 0.0
    w_up = np.zeros((E, m, d + 1))
    w_up[:, :, d] = 1.0
    w_down = rng.standard_normal((E, m, d + 1))
    mask = wl.bernoulli_mask(T, E, 0.6, seed=1)
    gated = oracle.expert_ffn(x, w_up, w_gate, None, w_down, None, mask, "gelu_erf", gated=True)
    plain = oracle.expert_ffn(x, w_gate, None, None, w_down, None, mask, "gelu_erf")
    np.testing.assert_allclose(gated, plain, rtol=0, atol=1e-13)


def test_single_expert_and_additivity(oracle):
    rng = np.random.default_rng(4)
    p = _small_layer(rng)
    T, E = 9, 5
    b2 = p["b_down"]
    singles = []
    for e in range(E):
        mask = np.zeros((T, E), np.uint8)
        mask[:, e] = 1
        y = _ffn(oracle, p, mask, "gelu_erf")
        h = p["x"] @ p["w_up"][e].T + p["b_up"][e]
        h = h * scipy.stats.norm.cdf(h)                       # GELU(v) = v * Phi(v)
        np.testing.assert_allclose(y - b2, h @ p["w_down"][e], rtol=0, atol=1e-12)
        singles.append(y - b2)
    a = wl.bernoulli_mask(T, E, 0.5, seed=2)
    b = (1 - a) * wl.bernoulli_mask(T, E, 0.5, seed=3)        # disjoint from a
    ya, yb, yab = (_ffn(oracle, p, mk, "gelu_erf") for mk in (a, b, a | b))
    np.testing.assert_allclose(yab - b2, (ya - b2) + (yb - b2), rtol=0, atol=1e-12)
    # a per-token mask is honoured token by token
    want = b2 + sum(a[:, [e]] * singles[e] for e in range(E))
    np.testing.assert_allclose(ya, want, rtol=0, atol=1e-12)


def test_empty_mask_gives_bias_or_zero(oracle):
    rng = np.random.default_rng(5)
    p = _small_layer(rng)
    z = np.zeros((9, 5), np.uint8)
    assert np.array_equal(_ffn(oracle, p, z, "relu"), np.tile(p["b_down"], (9, 1)))
    p["b_down"] = None
    assert not _ffn(oracle, p, z, "relu").any()


def test_activation_curves(oracle):
    v = np.linspace(-6, 6, 241)
    assert np.array_equal(_act_curve(oracle, "relu", v), np.maximum(v, 0))
    np.testing.assert_allclose(_act_curve(oracle, "gelu_erf", v), v * scipy.stats.norm.cdf(v),
                               rtol=0, atol=1e-14)
    tv = torch.from_numpy(v)
    np.testing.assert_allclose(_act_curve(oracle, "gelu_tanh", v),
                               torch.nn.functional.gelu(tv, approximate="tanh").numpy(),
                               rtol=0, atol=1e-14)
    # the two GELU forms are close but not equal: the activation code is part of the contract
    diff = np.abs(_act_curve(oracle, "gelu_erf", v) - _act_curve(oracle, "gelu_tanh", v)).max()
    assert 1e-5 < diff < 1e-3


def test_gated_bias_rejected(oracle):
    rng = np.random.default_rng(6)
    p = _small_layer(rng, gated=True, bias=False)
    with pytest.raises(RuntimeError):
        oracle.expert_ffn(p["x"], p["w_up"], p["w_gate"], np.zeros((5, 3)), p["w_down"], None,
                          np.ones((9, 5), np.uint8), "relu", gated=True)


def test_forward_tau_zero_is_dense_and_router_norm_meaning(oracle):
    """Whole layer on the tiny configuration: tau = 0 reproduces the dense FFN whatever the
    router says; and a single-expert mask yields the vector whose L2 norm the router is meant
    to predict (Sec. 3.3), which is what makes the unweighted sum the right merge."""
    cfg = wl.CONFIGS["cfg1"]
    layer, x = wl.make_layer(cfg, 0), wl.make_input(cfg, 0)
    y, s, mask = oracle.forward(layer, x, 0.0)
    assert mask.all()
    W1 = layer["w_up"].reshape(cfg.H, cfg.d)
    W2 = layer["w_down"].reshape(cfg.H, cfg.d)
    np.testing.assert_allclose(y, np.maximum(x @ W1.T, 0) @ W2, rtol=0, atol=1e-12)
    norms = np.stack([np.linalg.norm(np.maximum(x @ layer["w_up"][e].T, 0) @ layer["w_down"][e], axis=1)
                      for e in range(cfg.E)], axis=1)
    tot = np.zeros_like(y)
    for e in range(cfg.E):
        mk = np.zeros((cfg.T, cfg.E), np.uint8)
        mk[:, e] = 1
        ye = oracle.expert_ffn(x, layer["w_up"], None, None, layer["w_down"], None, mk, "relu")
        np.testing.assert_allclose(np.linalg.norm(ye, axis=1), norms[:, e], rtol=1e-12, atol=1e-14)
        tot += ye
    np.testing.assert_allclose(tot, y, rtol=0, atol=1e-12)
