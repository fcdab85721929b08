"""Seeded synthetic workloads shared by the oracle-side tests and the GPU-side tests / bench.

This module holds NO arithmetic of the method: it only draws random layers and inputs with the
shapes of the benchmark configurations, rounds them to the storage type and converts between
NumPy and the bf16 bit pattern.  Both the CPU oracle and the HIP library are fed from here so
that they see identical numbers.

All draws come from one numpy Generator(PCG64(seed)) in a fixed order: x first, then the layer
(w_up, w_gate, b_up, w_down, b_down, r_w1, r_b1, r_w2, r_b2).  Values are drawn in fp64, rounded
once to the storage type (round-to-nearest-even) and returned as fp64 arrays holding exactly
representable values.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

ACT_NAMES = ("relu", "gelu_erf", "gelu_tanh")


@dataclass(frozen=True)
class Config:
    name: str
    T: int            # tokens
    d: int            # model width
    E: int            # experts
    m: int            # neurons per expert
    d_h: int          # router hidden width
    gated: bool
    act: str          # one of ACT_NAMES
    dtype: str        # "f32" | "bf16": storage type of x, y and every parameter
    taus: tuple
    ffn_bias: bool = False      # draw b_up / b_down (std 0.02) instead of leaving them absent
    router_bias: bool = False   # draw r_b1 ~ N(0,1), r_b2 ~ N(0,0.25)
    row_scale: str = ""         # "lognormal": scale input rows by LogNormal(0,1)

    @property
    def H(self) -> int:
        return self.E * self.m


# The five benchmark configurations (numbered as in the benchmark description) plus the
# paper's own latency-experiment shape (Sec. 4.4: 24 experts of 128 neurons, 256x197 tokens).
CONFIGS = {
    "cfg1": Config("cfg1", 128, 64, 16, 16, 32, False, "relu", "f32", (0.0, 0.5, 0.9)),
    "cfg2": Config("cfg2", 128 * 128, 768, 128, 24, 128, False, "gelu_erf", "bf16",
                   (0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9), ffn_bias=True),
    "cfg3": Config("cfg3", 256 * 197, 768, 128, 24, 128, False, "gelu_erf", "bf16", (0.5,),
                   ffn_bias=True, router_bias=True, row_scale="lognormal"),
    "cfg4": Config("cfg4", 4096, 2048, 256, 64, 256, True, "gelu_tanh", "bf16", (0.3, 0.6)),
    "cfg5a": Config("cfg5a", 16, 2048, 256, 64, 256, True, "gelu_tanh", "bf16", (0.5,)),
    "cfg5b": Config("cfg5b", 16, 768, 32, 24, 128, False, "gelu_erf", "bf16", (0.5,),
                    ffn_bias=True),
    "paper": Config("paper", 256 * 197, 768, 24, 128, 128, False, "gelu_erf", "bf16", (0.5,),
                    ffn_bias=True),
    # the paper's own conversion of its language model (Sec. 4.3 / training details): 2048
    # experts of 8 neurons over the 16384-wide gated FFN, router hidden width 512
    "gemma_paper": Config("gemma_paper", 4096, 2048, 2048, 8, 512, True, "gelu_tanh", "bf16", (0.5,)),
    # the paper's own conversion of its text classifier (training details: expert size 6): 512
    # experts of 6 neurons over the 3072-wide FFN of a BERT-base layer
    "bert_paper": Config("bert_paper", 128 * 128, 768, 512, 6, 128, False, "gelu_erf", "bf16",
                         (0.5,), ffn_bias=True),
}


def with_tokens(cfg: Config, T: int) -> Config:
    return replace(cfg, T=int(T))


# ----------------------------------------------------------------------------- rounding

def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp64/fp32 values to bfloat16 (round-to-nearest-even), returned as fp64."""
    return bf16_bits_to_f64(f64_to_bf16_bits(a))


def f64_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) of the values, rounding fp64 -> fp32 -> bf16 (both RNE).

    Inputs here are drawn with far more than 24 significant bits, so the double rounding cannot
    land on a tie; finite values only."""
    f = np.ascontiguousarray(np.asarray(a, dtype=np.float64)).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = u + np.uint64(0x7FFF) + lsb
    return (u >> np.uint64(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(np.asarray(bits, dtype=np.uint16)).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def round_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round to the storage type and return fp64 holding the rounded values."""
    if dtype == "bf16":
        return round_bf16(a)
    if dtype == "f32":
        return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)
    raise ValueError(dtype)


def to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """Storage-typed NumPy array: float32, or uint16 bf16 bit patterns."""
    if dtype == "bf16":
        return f64_to_bf16_bits(a)
    if dtype == "f32":
        return np.ascontiguousarray(np.asarray(a, dtype=np.float64).astype(np.float32))
    raise ValueError(dtype)


def from_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return bf16_bits_to_f64(a)
    return np.asarray(a, dtype=np.float64)


# ----------------------------------------------------------------------------- draws

def make_input(cfg: Config, seed: int = 0) -> np.ndarray:
    """x[T, d] ~ N(0,1), optionally with LogNormal(0,1) row scales; rounded to cfg.dtype."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal((cfg.T, cfg.d))
    if cfg.row_scale == "lognormal":
        x = x * rng.lognormal(0.0, 1.0, size=(cfg.T, 1))
    elif cfg.row_scale:
        raise ValueError(cfg.row_scale)
    return round_storage(x, cfg.dtype)


def make_layer(cfg: Config, seed: int = 0) -> dict:
    """Random layer with weights ~ N(0, 1/fan_in), rounded to cfg.dtype, as fp64 arrays.

    Keys: w_up[E,m,d], w_gate[E,m,d] (gated only), b_up[E,m] or None, w_down[E,m,d],
    b_down[d] or None, r_w1[d_h,d], r_b1 or None, r_w2[E,d_h], r_b2 or None, act, gated."""
    # a different stream than make_input(seed) so that x and the layer are independent
    rng = np.random.Generator(np.random.PCG64([seed, 0x4D6F45]))
    E, m, d, dh, H = cfg.E, cfg.m, cfg.d, cfg.d_h, cfg.H
    rs = lambda a: round_storage(a, cfg.dtype)
    layer = {"act": cfg.act, "gated": cfg.gated}
    layer["w_up"] = rs(rng.standard_normal((E, m, d)) / np.sqrt(d))
    layer["w_gate"] = rs(rng.standard_normal((E, m, d)) / np.sqrt(d)) if cfg.gated else None
    if cfg.ffn_bias and not cfg.gated:
        layer["b_up"] = rs(0.02 * rng.standard_normal((E, m)))
    else:
        layer["b_up"] = None
    layer["w_down"] = rs(rng.standard_normal((E, m, d)) / np.sqrt(H))
    layer["b_down"] = rs(0.02 * rng.standard_normal((d,))) if cfg.ffn_bias else None
    layer["r_w1"] = rs(rng.standard_normal((dh, d)) / np.sqrt(d))
    layer["r_b1"] = rs(rng.standard_normal((dh,))) if cfg.router_bias else None
    layer["r_w2"] = rs(rng.standard_normal((E, dh)) / np.sqrt(dh))
    layer["r_b2"] = rs(0.5 * rng.standard_normal((E,))) if cfg.router_bias else None
    return layer


def bernoulli_mask(T: int, E: int, p, seed: int = 0) -> np.ndarray:
    """Gate decisions overridden by Bernoulli(p) draws (the device of Sec. 4.4 that controls
    the executed fraction independently of the router).  p is a scalar or a [T,1]/[T,E] array.
    Tokens with no expert at all can occur."""
    rng = np.random.Generator(np.random.PCG64([seed, 0xBE12]))
    return (rng.random((T, E)) < np.asarray(p)).astype(np.uint8)


def random_scores(T: int, E: int, seed: int = 0, kind: str = "halfnormal") -> np.ndarray:
    """fp32-representable non-negative score tables for select tests (returned as float32)."""
    rng = np.random.Generator(np.random.PCG64([seed, 0x5C0]))
    if kind == "halfnormal":
        s = np.abs(rng.standard_normal((T, E)))
    elif kind == "grid":          # many exact ties and exact-threshold hits
        s = rng.integers(0, 9, size=(T, E)).astype(np.float64) * 0.25
    elif kind == "zipf":          # a few hot experts
        s = np.abs(rng.standard_normal((T, E))) * (1.0 / (1.0 + np.arange(E)))[None, :] ** 0.7
    else:
        raise ValueError(kind)
    return np.ascontiguousarray(s.astype(np.float32))


def quantize_experts_e4m3(layer: dict) -> dict:
    """The layer with its expert matrices stored in 8-bit floating point (OCP E4M3: 4 exponent
    bits, 3 mantissa bits, largest value 448) with one power-of-two scale per expert and matrix,
    chosen so that the largest weight of the matrix just fits.  Returns a copy whose w_up / w_gate
    / w_down hold the DEQUANTISED values as fp64 (each exactly a bf16 number), so that the oracle
    sees the numbers the library computes with, plus "w8": the uint8 codes [E, m, d] and the
    float32 scales [E, 3] (up, gate, down) that the library is given.  Rounding to the format is
    storage rounding like the bf16 rounding above, done by torch's float8_e4m3fn cast (round to
    nearest even)."""
    import torch
    out = dict(layer)
    E = layer["w_up"].shape[0]
    scales = np.ones((E, 3), np.float32)
    w8 = {}
    for which, key in enumerate(("w_up", "w_gate", "w_down")):
        w = layer.get(key)
        if w is None:
            w8[key] = None
            continue
        amax = np.abs(w).reshape(E, -1).max(axis=1)
        s = np.exp2(np.ceil(np.log2(np.maximum(amax, 1e-30) / 448.0)))
        scales[:, which] = s
        q = torch.from_numpy((w / s[:, None, None]).astype(np.float32)).to(torch.float8_e4m3fn)
        w8[key] = q.view(torch.uint8).numpy().copy()
        out[key] = q.to(torch.float32).numpy().astype(np.float64) * s[:, None, None]
    w8["scales"] = scales
    out["w8"] = w8
    return out
