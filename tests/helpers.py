"""Shared pieces of the GPU parity tests: error metrics and oracle-side conveniences."""
import numpy as np

from paper_2310_04361_amd import workloads as wl

TOL = {"bf16": 2e-2, "f32": 1e-5}


def tokenwise_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max over tokens of ||got_t - ref_t||_inf / ||ref_t||_inf (rows with ref_t = 0 must match
    to 1e-30 absolutely)."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    if got.size == 0:
        return 0.0
    num = np.abs(got - ref).max(axis=1)
    den = np.abs(ref).max(axis=1)
    zero = den == 0
    assert (num[zero] <= 1e-30).all()
    return float((num[~zero] / den[~zero]).max()) if (~zero).any() else 0.0


def elementwise_rel_err(got: np.ndarray, ref: np.ndarray, eps: float = 1e-3) -> float:
    """max over all elements of |got - ref| / (|ref| + eps * ||ref_t||_inf): the element-wise
    companion of tokenwise_rel_err (reported next to it; eps keeps near-zero outputs, whose
    error is the rounding noise of the whole sum, from dividing by nothing)."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    if got.size == 0:
        return 0.0
    den = np.abs(ref) + eps * np.abs(ref).max(axis=1, keepdims=True)
    ok = den > 0
    return float((np.abs(got - ref)[ok] / den[ok]).max()) if ok.any() else 0.0


def lists_from_mask(mask: np.ndarray, shuffle_seed=None):
    """Expert-major lists (offsets[E+1], token_lists[P]) of a 0/1 mask, optionally with each
    expert's list shuffled (the order inside a list is not part of the contract)."""
    T, E = mask.shape
    rng = np.random.default_rng(shuffle_seed) if shuffle_seed is not None else None
    lists, offsets = [], [0]
    for e in range(E):
        tok = np.flatnonzero(mask[:, e]).astype(np.int32)
        if rng is not None:
            rng.shuffle(tok)
        lists.append(tok)
        offsets.append(offsets[-1] + len(tok))
    flat = np.concatenate(lists) if lists else np.zeros(0, np.int32)
    return np.asarray(offsets, np.int32), flat.astype(np.int32)


def oracle_ffn(oracle, layer, x, mask, quantize_h=False):
    return oracle.expert_ffn(x, layer["w_up"], layer.get("w_gate"), layer.get("b_up"),
                             layer["w_down"], layer.get("b_down"), mask, layer["act"],
                             gated=bool(layer.get("gated")), quantize_h=quantize_h)


def small_cfg(name, T, E=None):
    """A benchmark configuration at a test-sized token count (and optionally fewer experts,
    which keeps every per-expert shape the kernels see)."""
    from dataclasses import replace
    cfg = wl.with_tokens(wl.CONFIGS[name], T)
    return replace(cfg, E=E) if E else cfg


def tokenwise_rel_errs(y, y_ref):
    """Per-token ||y_t - ref_t||_inf / ||ref_t||_inf (the vector whose maximum tokenwise_rel_err is)."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    den = np.abs(y_ref).max(axis=1)
    den = np.where(den > 0, den, 1.0)
    return np.abs(y - y_ref).max(axis=1) / den


def quantised_hidden_row(oracle, layer, xq_t, e):
    """The oracle's quantised hidden row of (token, expert e), read out through the oracle itself:
    one token, one expert, and a down matrix that copies neuron j to output column j."""
    m, d = layer["w_up"].shape[1], layer["w_up"].shape[2]
    ident = np.zeros((1, m, d))
    ident[0, np.arange(m), np.arange(m)] = 1.0
    y = oracle.expert_ffn(xq_t[None, :], layer["w_up"][e:e + 1],
                          layer["w_gate"][e:e + 1] if layer.get("gated") else None,
                          layer["b_up"][e:e + 1] if layer.get("b_up") is not None else None,
                          ident, None, np.ones((1, 1), np.uint8), layer["act"],
                          gated=bool(layer.get("gated")), quantize_h=True)
    return y[0, :m]


def check_fully_8bit(oracle, layer, xq, mask, got, ref, tol, max_share=0.01):
    """Bar for layers with 8-bit hidden activations.  A hidden activation that the GPU computes a
    hair differently from the oracle (the 8-bit matrix instruction adds a block's products with
    less than fp32 precision) can fall on the other side of a rounding boundary and take the
    neighbouring E4M3 value: one step of that element, which for a token with few experts is more
    than the bf16 bar.  Every token must meet `tol`, or exceed it by no more than two such
    single-step differences of its own hidden rows (the largest |step * W_down row| relative to
    the token's output, from the oracle's quantised rows); at most `max_share` of the tokens may
    need that allowance.  Returns (largest error, tokens that used the allowance)."""
    errs = tokenwise_rel_errs(got, ref)
    over = np.nonzero(errs > tol)[0]
    assert len(over) <= max_share * len(errs) + 1, f"{len(over)} of {len(errs)} tokens exceed {tol}"
    w_down = np.asarray(layer["w_down"], dtype=np.float64)
    for t in over:
        budget = 0.0
        for e in np.nonzero(mask[t])[0]:
            hq = quantised_hidden_row(oracle, layer, np.asarray(xq[t], dtype=np.float64), int(e))
            nz = hq != 0
            step = np.zeros_like(hq)
            step[nz] = 2.0 * np.exp2(np.floor(np.log2(np.abs(hq[nz]))) - 3)
            budget = max(budget, float((step * np.abs(w_down[e]).max(axis=1)).max()))
        budget /= max(np.abs(ref[t]).max(), 1e-300)
        assert errs[t] <= tol + 2 * budget, (int(t), float(errs[t]), budget)
    return float(errs.max()) if len(errs) else 0.0, len(over)
