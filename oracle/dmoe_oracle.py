"""ctypes front end of the fp64 CPU oracle (dmoe_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's cpu_baseline
leg.  It never imports the HIP package and the HIP package never imports it.

Every function takes array-likes, converts them to contiguous fp64 and returns NumPy arrays.
The caller rounds inputs to the storage type (bf16 / fp32) beforehand.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dmoe_oracle.c")
_LIB_DIR = os.path.join(_HERE, "_build")
_LIB = os.path.join(_LIB_DIR, "libdmoe_oracle.so")

ACT_RELU, ACT_GELU_ERF, ACT_GELU_TANH = 0, 1, 2
ACT_BY_NAME = {"relu": ACT_RELU, "gelu_erf": ACT_GELU_ERF, "gelu_tanh": ACT_GELU_TANH}

_lib = None


def build(force: bool = False) -> str:
    """Compile dmoe_oracle.c with gcc (OpenMP) into oracle/_build/."""
    os.makedirs(_LIB_DIR, exist_ok=True)
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB + ".tmp", _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(_LIB + ".tmp", _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        i32p = ctypes.POINTER(ctypes.c_int32)
        ci = ctypes.c_int
        lib.dmoe_oracle_num_threads.restype = ci
        lib.dmoe_oracle_router.argtypes = [dp, dp, dp, dp, dp, ci, ci, ci, ci, dp]
        lib.dmoe_oracle_select.argtypes = [dp, ci, ci, ctypes.c_double, u8p, i32p]
        lib.dmoe_oracle_select_topk.argtypes = [dp, ci, ci, ci, u8p]
        lib.dmoe_oracle_bucket.argtypes = [u8p, ci, ci, i32p, i32p, i32p]
        lib.dmoe_oracle_expert_ffn.argtypes = [dp, dp, dp, dp, dp, dp, ci, ci, ci, ci, ci, ci,
                                               u8p, dp]
        lib.dmoe_oracle_quantize_rows_e4m3.argtypes = [dp, ci, ci, dp, dp]
        lib.dmoe_oracle_quantize_rows_e4m3.restype = ci
        lib.dmoe_oracle_expert_ffn_q8h.argtypes = lib.dmoe_oracle_expert_ffn.argtypes
        lib.dmoe_oracle_expert_ffn_q8h.restype = ci
        lib.dmoe_oracle_round_bf16.argtypes = [dp, ctypes.c_size_t, dp]
        lib.dmoe_oracle_round_bf16.restype = ci
        for f in (lib.dmoe_oracle_router, lib.dmoe_oracle_select, lib.dmoe_oracle_select_topk,
                  lib.dmoe_oracle_bucket, lib.dmoe_oracle_expert_ffn):
            f.restype = ci
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().dmoe_oracle_num_threads())


def _f64(a, shape=None):
    if a is None:
        return None
    a = np.ascontiguousarray(np.asarray(a, dtype=np.float64))
    if shape is not None and a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _dp(a):
    if a is None:
        return ctypes.POINTER(ctypes.c_double)()
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def router(x, r_w1, r_b1, r_w2, r_b2):
    """scores[T, E] = | r_w2 @ relu(r_w1 @ x_t + r_b1) + r_b2 |  (Sec. 3.3)."""
    x = _f64(x)
    T, d = x.shape
    r_w1 = _f64(r_w1)
    dh = r_w1.shape[0]
    r_w1 = _f64(r_w1, (dh, d))
    r_w2 = _f64(r_w2)
    E = r_w2.shape[0]
    r_w2 = _f64(r_w2, (E, dh))
    r_b1 = _f64(r_b1, (dh,)) if r_b1 is not None else None
    r_b2 = _f64(r_b2, (E,)) if r_b2 is not None else None
    scores = np.empty((T, E), dtype=np.float64)
    rc = _load().dmoe_oracle_router(_dp(x), _dp(r_w1), _dp(r_b1), _dp(r_w2), _dp(r_b2),
                                    T, d, dh, E, _dp(scores))
    if rc:
        raise RuntimeError(f"dmoe_oracle_router failed: {rc}")
    return scores


def select(scores, tau):
    """Dynamic-k gate (Eq. 4).  tau is used as given: pass float(np.float32(tau)) to mirror a
    C float argument.  Returns (mask uint8 [T, E], k_per_token int32 [T])."""
    scores = _f64(scores)
    T, E = scores.shape
    mask = np.empty((T, E), dtype=np.uint8)
    k = np.empty((T,), dtype=np.int32)
    rc = _load().dmoe_oracle_select(_dp(scores), T, E, float(tau),
                                    mask.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
                                    k.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    if rc:
        raise RuntimeError(f"dmoe_oracle_select failed: {rc}")
    return mask, k


def select_topk(scores, k):
    """Top-k gate: the k largest scores per token, ties towards the lower expert index."""
    scores = _f64(scores)
    T, E = scores.shape
    mask = np.empty((T, E), dtype=np.uint8)
    rc = _load().dmoe_oracle_select_topk(_dp(scores), T, E, int(k),
                                         mask.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)))
    if rc:
        raise RuntimeError(f"dmoe_oracle_select_topk failed: {rc}")
    return mask


def bucket(mask):
    """Per-expert token lists: returns (counts[E], offsets[E+1], token_lists[P]) int32."""
    mask = np.ascontiguousarray(np.asarray(mask, dtype=np.uint8))
    T, E = mask.shape
    counts = np.empty((E,), dtype=np.int32)
    offsets = np.empty((E + 1,), dtype=np.int32)
    lists = np.empty((max(T * E, 1),), dtype=np.int32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    rc = _load().dmoe_oracle_bucket(mask.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), T, E,
                                    counts.ctypes.data_as(i32p), offsets.ctypes.data_as(i32p),
                                    lists.ctypes.data_as(i32p))
    if rc:
        raise RuntimeError(f"dmoe_oracle_bucket failed: {rc}")
    return counts, offsets, lists[: int(offsets[E])].copy()


def expert_ffn(x, w_up, w_gate, b_up, w_down, b_down, mask, act, gated=False, quantize_h=False):
    """y[T, d] = b_down + sum of the selected experts' outputs (Sec. 3.2, Appendix G).

    w_up / w_gate / w_down are expert-major [E, m, d]; b_up [E, m] or None; b_down [d] or None;
    mask [T, E] of 0/1; act is an ACT_* code or its name.  quantize_h: every selected
    (token, expert) row of hidden activations is rounded to bfloat16 and then quantised to E4M3
    with a power-of-two row scale before the down-projection (the fully 8-bit layers)."""
    if isinstance(act, str):
        act = ACT_BY_NAME[act]
    x = _f64(x)
    T, d = x.shape
    w_up = _f64(w_up)
    E, m, _ = w_up.shape
    w_up = _f64(w_up, (E, m, d))
    w_down = _f64(w_down, (E, m, d))
    w_gate = _f64(w_gate, (E, m, d)) if gated else None
    b_up = _f64(b_up, (E, m)) if b_up is not None else None
    b_down = _f64(b_down, (d,)) if b_down is not None else None
    mask = np.ascontiguousarray(np.asarray(mask, dtype=np.uint8))
    if mask.shape != (T, E):
        raise ValueError(f"mask must be {(T, E)}, got {mask.shape}")
    y = np.empty((T, d), dtype=np.float64)
    fn = _load().dmoe_oracle_expert_ffn_q8h if quantize_h else _load().dmoe_oracle_expert_ffn
    rc = fn(_dp(x), _dp(w_up), _dp(w_gate), _dp(b_up), _dp(w_down), _dp(b_down), T, d, E, m,
            1 if gated else 0, int(act), mask.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), _dp(y))
    if rc:
        raise RuntimeError(f"dmoe_oracle_expert_ffn failed: {rc}")
    return y


def round_bf16(v):
    """Nearest bfloat16 numbers (ties to even) of an array, as fp64."""
    v = _f64(v)
    out = np.empty_like(v)
    rc = _load().dmoe_oracle_round_bf16(_dp(v), ctypes.c_size_t(v.size), _dp(out))
    if rc:
        raise RuntimeError(f"dmoe_oracle_round_bf16 failed: {rc}")
    return out


def quantize_rows_e4m3(x):
    """Row-wise 8-bit (E4M3, power-of-two scale per row) quantisation of the experts' input.
    Returns (xq[T, d] -- the quantised rows as fp64 numbers --, scales[T])."""
    x = _f64(x)
    T, d = x.shape
    xq = np.empty((T, d), dtype=np.float64)
    scales = np.empty((T,), dtype=np.float64)
    rc = _load().dmoe_oracle_quantize_rows_e4m3(_dp(x), T, d, _dp(xq), _dp(scales))
    if rc:
        raise RuntimeError(f"dmoe_oracle_quantize_rows_e4m3 failed: {rc}")
    return xq, scales


def forward(layer: dict, x, tau):
    """Whole layer on fp64 copies of `layer` (a dict with the keys of workloads.make_layer).
    Returns (y, scores, mask)."""
    s = router(x, layer["r_w1"], layer.get("r_b1"), layer["r_w2"], layer.get("r_b2"))
    mask, _ = select(s, tau)
    y = expert_ffn(x, layer["w_up"], layer.get("w_gate"), layer.get("b_up"), layer["w_down"],
                   layer.get("b_down"), mask, layer["act"], gated=bool(layer.get("gated", False)))
    return y, s, mask
