"""Pins for the oracle's router (Sec. 3.3): a hand-worked example, the special case that is a
pair of library matrix products, and a distributional closed form."""
import numpy as np

from paper_2310_04361_amd import workloads as wl


def test_hand_worked_example(oracle):
    # x = (1, -2); hidden pre-activations: (1*1 + 0.5*-2 + 0.25, -1*1 + 1*-2 + 0) = (0.25, -3)
    # relu -> (0.25, 0); outputs: (4*0.25 + 9*0 - 2, -8*0.25 + 9*0 + 0.5, 0 + 0 - 0.125)
    #       = (-1, -1.5, -0.125) -> abs -> (1, 1.5, 0.125)
    x = [[1.0, -2.0]]
    r_w1 = [[1.0, 0.5], [-1.0, 1.0]]
    r_b1 = [0.25, 0.0]
    r_w2 = [[4.0, 9.0], [-8.0, 9.0], [0.0, 0.0]]
    r_b2 = [-2.0, 0.5, -0.125]
    s = oracle.router(x, r_w1, r_b1, r_w2, r_b2)
    assert s.tolist() == [[1.0, 1.5, 0.125]]
    # without biases: hidden (0, 0) since 1 - 1 = 0 and -3 < 0 -> all scores 0
    s0 = oracle.router(x, r_w1, None, r_w2, None)
    assert s0.tolist() == [[0.0, 0.0, 0.0]]


def test_against_library_matmul(oracle):
    rng = np.random.default_rng(0)
    T, d, dh, E = 33, 19, 7, 11          # all different: a transposed operand cannot pass
    x = rng.standard_normal((T, d))
    r_w1, r_b1 = rng.standard_normal((dh, d)), rng.standard_normal(dh)
    r_w2, r_b2 = rng.standard_normal((E, dh)), rng.standard_normal(E)
    ref = np.abs(np.maximum(x @ r_w1.T + r_b1, 0.0) @ r_w2.T + r_b2)
    got = oracle.router(x, r_w1, r_b1, r_w2, r_b2)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    assert (got >= 0).all()
    ref0 = np.abs(np.maximum(x @ r_w1.T, 0.0) @ r_w2.T)
    np.testing.assert_allclose(oracle.router(x, r_w1, None, r_w2, None), ref0, rtol=0, atol=1e-12)


def test_positive_homogeneity_without_biases(oracle):
    """relu and abs are positively homogeneous: scaling an input row by 2^k scales its scores
    by exactly 2^k, hence the gate (Eq. 4) cannot depend on the row's scale."""
    cfg = wl.with_tokens(wl.CONFIGS["cfg1"], 40)
    layer, x = wl.make_layer(cfg, 1), wl.make_input(cfg, 1)
    s = oracle.router(x, layer["r_w1"], None, layer["r_w2"], None)
    s8 = oracle.router(x * 8.0, layer["r_w1"], None, layer["r_w2"], None)
    assert np.array_equal(s8, 8.0 * s)
    tau = float(np.float32(0.5))
    assert np.array_equal(oracle.select(s, tau)[0], oracle.select(s8, tau)[0])


def test_selected_fraction_matches_half_normal_law(oracle):
    """With zero biases and Gaussian second-layer rows, a token's scores are, given its hidden
    vector, i.i.d. half-normal up to one common scale.  So the mean fraction of experts kept by
    Eq. 4 equals that of |z_i| >= tau max|z| for z i.i.d. N(0,1), whatever x is."""
    E, dh, d, T = 64, 128, 48, 1500
    rng = np.random.default_rng(7)
    x = rng.standard_normal((T, d))
    r_w1 = rng.standard_normal((dh, d)) / np.sqrt(d)
    r_w2 = rng.standard_normal((E, dh)) / np.sqrt(dh)
    s = oracle.router(x, r_w1, None, r_w2, None)
    z = np.abs(np.random.default_rng(8).standard_normal((40000, E)))
    for tau in (0.3, 0.5, 0.8):
        kept = oracle.select(s, tau)[0].mean()
        law = (z >= tau * z.max(axis=1, keepdims=True)).mean()
        # one layer draw: the scores of different tokens share r_w2, so allow a wide band
        assert abs(kept - law) < 0.02 + 0.1 * law, (tau, kept, law)
