"""MI355X-native dynamic-k Mixture-of-Experts FFN forward (D2DMoE inference hot path).

`paper_2310_04361_amd.binding` wraps the C-ABI library built from `csrc/` (loaded lazily, so
that `workloads` and `cost_model` can be imported on a machine without the built library).
"""

__all__ = ["binding", "workloads", "cost_model"]
