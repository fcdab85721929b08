"""Pins of the oracle's row-wise E4M3 quantiser (the 8-bit expert input of the lower-precision
layers, Appendix C).  The format -- OCP 8-bit floating point E4M3: 1 sign, 4 exponent bits with
bias 7, 3 mantissa bits, subnormals m/8 * 2^-6, no infinities, largest value 448 -- is written
out here from its definition, and torch's float8_e4m3fn cast serves as an independent converter."""
import numpy as np
import pytest


def e4m3_values():
    """All non-negative finite E4M3 values, ascending, with their codes (from the definition)."""
    vals = []
    for code in range(0x7f):                       # 0x7f is NaN
        e, m = code >> 3, code & 7
        vals.append((m / 8.0 * 2.0 ** -6) if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7))
    assert vals == sorted(vals) and vals[-1] == 448.0 and vals[1] == 2.0 ** -9
    return np.asarray(vals)


def test_representable_values_are_fixed_points(oracle):
    v = e4m3_values()
    for k in (-20, -3, 0, 5, 31):
        s = 2.0 ** k
        row = np.concatenate([v, -v, [448.0]]) * s            # the row maximum is 448 s
        xq, scales = oracle.quantize_rows_e4m3(row[None, :])
        assert scales[0] == s
        assert np.array_equal(xq[0], row)


def test_midpoints_go_to_the_even_mantissa_and_neighbours_round_to_nearest(oracle):
    v = e4m3_values()
    mid = (v[:-1] + v[1:]) / 2
    even = np.where(np.arange(len(v) - 1) % 2 == 0, v[:-1], v[1:])   # code parity = mantissa parity
    row = np.concatenate([mid, [448.0]])
    xq, _ = oracle.quantize_rows_e4m3(np.stack([row, -row]))
    assert np.array_equal(xq[0, :-1], even) and np.array_equal(xq[1, :-1], -even)
    # a hair below / above a midpoint goes down / up
    lo = np.concatenate([mid * (1 - 2.0 ** -30), [448.0]])
    hi = np.concatenate([mid * (1 + 2.0 ** -30), [448.0]])
    xq, _ = oracle.quantize_rows_e4m3(np.stack([lo, hi]))
    assert np.array_equal(xq[0, :-1], v[:-1]) and np.array_equal(xq[1, :-1], v[1:])


def test_scale_is_the_smallest_power_of_two_that_fits(oracle):
    rows = np.zeros((6, 8))
    rows[0, 3] = 448.0                 # fits with s = 1
    rows[1, 3] = -448.0 * (1 + 2.0 ** -20)   # just above: s = 2
    rows[2, 0] = 224.0                 # s = 0.5 would give exactly 448
    rows[3, 5] = 448.0 * 2.0 ** -40
    rows[4, 1] = 3.0                   # 3 / 448 = 0.0067 -> s = 2^-7 (0.0078)
    xq, s = oracle.quantize_rows_e4m3(rows)
    assert s.tolist() == [1.0, 2.0, 0.5, 2.0 ** -40, 2.0 ** -7, 1.0]
    assert np.array_equal(xq[5], np.zeros(8))            # a zero row stays zero, scale 1
    assert xq[1, 3] == -448.0                            # 224.0001.. * 2 -> nearest value
    # every row's largest element lands in (224, 448] in units of its scale
    rng = np.random.default_rng(0)
    x = rng.standard_normal((50, 64)) * np.exp(rng.normal(0, 4, (50, 1)))
    _, s = oracle.quantize_rows_e4m3(x)
    top = np.abs(x).max(axis=1) / s
    assert ((top > 224.0) & (top <= 448.0)).all()
    assert np.array_equal(np.log2(s), np.round(np.log2(s)))


def test_power_of_two_row_scaling_moves_only_the_scale(oracle):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((20, 96))
    xq, s = oracle.quantize_rows_e4m3(x)
    xq2, s2 = oracle.quantize_rows_e4m3(x * 2.0 ** 11)
    assert np.array_equal(s2, s * 2.0 ** 11) and np.array_equal(xq2, xq * 2.0 ** 11)


def test_against_an_independent_converter_and_the_half_step_bound(oracle):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(2)
    x = rng.standard_normal((64, 256)) * np.exp(rng.normal(0, 2, (64, 1)))
    x = x.astype(np.float32).astype(np.float64)
    xq, s = oracle.quantize_rows_e4m3(x)
    cast = torch.from_numpy((x / s[:, None]).astype(np.float32)).to(torch.float8_e4m3fn)
    ref = cast.to(torch.float32).numpy().astype(np.float64) * s[:, None]
    assert np.array_equal(xq, ref)
    # nearest value: the error is at most half a grid step (2^-4 relative, 2^-10 s absolute below 2^-6 s)
    err = np.abs(xq - x)
    bound = np.maximum(np.abs(x) * 2.0 ** -4, s[:, None] * 2.0 ** -10)
    assert (err <= bound).all()


# ---- 8-bit hidden activations (oracle.expert_ffn(..., quantize_h=True)) ---------------------------

def test_bf16_rounding_against_an_independent_converter_and_ties(oracle):
    import torch
    rng = np.random.default_rng(7)
    v = np.concatenate([rng.standard_normal(4000) * np.exp(rng.normal(0, 6, 4000)), [0.0, -0.0]])
    got = oracle.round_bf16(v)
    ref = torch.from_numpy(v.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    # (the fp32 step in between cannot move a value across a bf16 midpoint unless it sits within
    # 2^-16 of it: none of these draws does)
    assert np.array_equal(got, ref)
    # exact ties: 1 + 2^-8 lies half-way between 1 and 1 + 2^-7 (mantissa 0000000 is even);
    # 1 + 3 * 2^-8 half-way between 1 + 2^-7 (odd) and 1 + 2^-6 (even)
    assert oracle.round_bf16(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -(1 + 2.0 ** -8)])).tolist() == \
        [1.0, 1 + 2.0 ** -6, -1.0]


def _relu_layer(w_up, w_down):
    return dict(w_up=np.asarray(w_up, float), w_gate=None, b_up=None, w_down=np.asarray(w_down, float),
                b_down=None, act="relu", gated=False)


def _ffn(oracle, layer, x, mask, quantize_h):
    return oracle.expert_ffn(x, layer["w_up"], layer["w_gate"], layer["b_up"], layer["w_down"],
                             layer["b_down"], mask, layer["act"], layer["gated"], quantize_h=quantize_h)


def test_hidden_rows_of_small_integers_pass_unchanged(oracle):
    """Integers up to 15 have four significant bits: whatever power-of-two scale the row gets,
    they are E4M3 numbers, so the 8-bit-hidden result equals the plain one exactly."""
    rng = np.random.default_rng(1)
    E, m, d, T = 3, 5, 4, 7
    w_up = rng.integers(-2, 3, size=(E, m, d))
    x = rng.integers(0, 2, size=(T, d)).astype(float)       # h = relu(w x): integers in 0 .. 8
    w_down = rng.standard_normal((E, m, d))
    mask = rng.integers(0, 2, size=(T, E)).astype(np.uint8)
    layer = _relu_layer(w_up, w_down)
    assert np.array_equal(_ffn(oracle, layer, x, mask, True), _ffn(oracle, layer, x, mask, False))


def test_hand_worked_hidden_row(oracle):
    """One token, one expert of two neurons with h = (17, 1): the row maximum 17 gives the scale
    2^-4 (17 / 448 = 0.038 needs 2^-4), 17 / 2^-4 = 272 lies half-way between the E4M3 numbers
    256 and 288 and goes to the even mantissa, 256, so the 17 becomes 16; the 1 stays.
    y = 16 * w_down[0] + 1 * w_down[1]."""
    layer = _relu_layer([[[17.0, 0.0], [0.0, 1.0]]], [[[1.0, 10.0], [100.0, 1000.0]]])
    x = np.array([[1.0, 1.0]])
    mask = np.ones((1, 1), np.uint8)
    assert _ffn(oracle, layer, x, mask, False).tolist() == [[17.0 + 100.0, 170.0 + 1000.0]]
    assert _ffn(oracle, layer, x, mask, True).tolist() == [[16.0 + 100.0, 160.0 + 1000.0]]
    # ... and an unselected expert contributes nothing, quantised or not
    assert _ffn(oracle, layer, x, np.zeros((1, 1), np.uint8), True).tolist() == [[0.0, 0.0]]


def test_recomposed_from_the_pinned_pieces(oracle):
    """Gated GELU experts: hidden rows by NumPy and torch, rounded to bf16 by torch, quantised
    by the (pinned) row quantiser, multiplied out by NumPy -- the same result as the oracle's
    one-call path."""
    import torch
    rng = np.random.default_rng(3)
    E, m, d, T = 4, 6, 16, 9
    w_up, w_gate, w_down = (rng.standard_normal((E, m, d)) for _ in range(3))
    x = rng.standard_normal((T, d))
    mask = rng.integers(0, 2, size=(T, E)).astype(np.uint8)
    mask[0] = 1
    got = oracle.expert_ffn(x, w_up, w_gate, None, w_down, None, mask, "gelu_tanh", True, quantize_h=True)
    ref = np.zeros((T, d))
    for t in range(T):
        for e in range(E):
            if not mask[t, e]:
                continue
            g = torch.nn.functional.gelu(torch.from_numpy(w_gate[e] @ x[t]), approximate="tanh").numpy()
            h = g * (w_up[e] @ x[t])
            h16 = torch.from_numpy(h.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
            hq, _ = oracle.quantize_rows_e4m3(h16[None, :])
            ref[t] += hq[0] @ w_down[e]
    assert np.allclose(got, ref, rtol=0, atol=1e-12 * np.abs(ref).max())
    # the quantisation is visible against the unquantised layer
    plain = oracle.expert_ffn(x, w_up, w_gate, None, w_down, None, mask, "gelu_tanh", True)
    assert np.abs(got - plain).max() > 1e-3 * np.abs(plain).max()


def test_the_one_step_allowance_accepts_a_planted_step_and_rejects_more(oracle):
    """The bar for 8-bit hidden activations (helpers.check_fully_8bit) on the CPU: a result that
    differs from the oracle's by ONE E4M3 step of one hidden activation passes although it misses
    the plain tolerance; five steps on the same activation, or a one-step difference on every
    token, do not."""
    from helpers import check_fully_8bit, oracle_ffn, quantised_hidden_row
    rng = np.random.default_rng(5)
    E, m, d, T = 3, 8, 16, 40
    layer = dict(w_up=rng.standard_normal((E, m, d)), w_gate=rng.standard_normal((E, m, d)), b_up=None,
                 w_down=rng.standard_normal((E, m, d)), b_down=None, act="gelu_tanh", gated=True)
    x = rng.standard_normal((T, d))
    xq, _ = oracle.quantize_rows_e4m3(x)
    mask = np.zeros((T, E), np.uint8)
    mask[:, 1] = 1                                   # one expert per token: a step weighs most
    ref = oracle_ffn(oracle, layer, xq, mask, quantize_h=True)
    # token 7: its largest hidden activation one E4M3 step up (the spacing at that magnitude)
    hq = quantised_hidden_row(oracle, layer, xq[7], 1)
    j = int(np.abs(hq).argmax())
    step = np.exp2(np.floor(np.log2(abs(hq[j]))) - 3)
    tol = 1e-3
    planted = ref.copy()
    planted[7] += step * layer["w_down"][1, j]
    assert np.abs(planted[7] - ref[7]).max() / np.abs(ref[7]).max() > tol      # misses the plain bar
    err, n_allow = check_fully_8bit(oracle, layer, xq, mask, planted, ref, tol, max_share=0.05)
    assert n_allow == 1 and err > tol
    worse = ref.copy()
    worse[7] += 5 * step * layer["w_down"][1, j]
    with pytest.raises(AssertionError):
        check_fully_8bit(oracle, layer, xq, mask, worse, ref, tol, max_share=0.05)
    everywhere = ref.copy()
    for t in range(T):
        everywhere[t] += 0.01 * np.abs(ref[t]).max()
    with pytest.raises(AssertionError):              # too many tokens would need the allowance
        check_fully_8bit(oracle, layer, xq, mask, everywhere, ref, tol, max_share=0.05)
