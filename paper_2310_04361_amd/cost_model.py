"""FLOPs accounting of the layer (Appendix B), used by the benchmark.

The paper counts one operation per multiply-accumulate: C_FFN = 2 e d_m^2, C_E = C_FFN / n,
C_R = d_m d_h + d_h n.  Throughput figures here use the usual 2 FLOPs per multiply-accumulate
and say so; the ratio below is independent of that convention.
"""
from __future__ import annotations


def dense_ffn_macs(d: int, H: int, gated: bool = False) -> int:
    """Multiply-accumulates of the dense FFN per token: up (+gate) and down projections."""
    return (3 if gated else 2) * d * H


def expert_macs(d: int, m: int, gated: bool = False) -> int:
    """Multiply-accumulates of one expert for one token (C_E of Appendix B)."""
    return (3 if gated else 2) * d * m


def router_macs(d: int, d_h: int, E: int) -> int:
    """C_R of Appendix B."""
    return d * d_h + d_h * E


def cost_ratio(k: float, d: int, E: int, m: int, d_h: int, gated: bool = False) -> float:
    """C_dynk / C_FFN = k/n + C_R / C_FFN for k executed experts per token."""
    return (k * expert_macs(d, m, gated) + router_macs(d, d_h, E)) / dense_ffn_macs(d, E * m, gated)


def executed_flops(pairs: int, d: int, m: int, gated: bool = False) -> float:
    """FLOPs (2 per multiply-accumulate) of `pairs` executed (token, expert) pairs."""
    return 2.0 * pairs * expert_macs(d, m, gated)
