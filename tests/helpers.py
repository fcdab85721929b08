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


def oracle_ffn(oracle, layer, x, mask):
    return oracle.expert_ffn(x, layer["w_up"], layer.get("w_gate"), layer.get("b_up"),
                             layer["w_down"], layer.get("b_down"), mask, layer["act"],
                             gated=bool(layer.get("gated")))


def small_cfg(name, T, E=None):
    """A benchmark configuration at a test-sized token count (and optionally fewer experts,
    which keeps every per-expert shape the kernels see)."""
    from dataclasses import replace
    cfg = wl.with_tokens(wl.CONFIGS[name], T)
    return replace(cfg, E=E) if E else cfg
