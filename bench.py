#!/usr/bin/env python3
"""Benchmark of the dynamic-k MoE FFN forward on one MI355X.

One step = one dmoe_forward (router, gate, bucketing, experts) over one batch of synthetic
tokens that already sit in HBM.  The headline workload is the BERT-base-shaped bf16 layer
(d=768, 128 experts of 24 neurons, GELU, 128x128 tokens) at tau = 0.5.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2] [--tau 0.5] [--sweep]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 matrix peak
# HBM bytes per launch of the dominant kernel from separate `rocprofv3 --pmc FETCH_SIZE` /
# `WRITE_SIZE` runs of this script, scaled by the same counters' readings for a plain 256 MiB copy
# (profiles/dmoe_forward_cfg2_tau0.5_hbm_traffic.txt).  Only valid for the exact workload named.
MEASURED_TRAFFIC = {("cfg2", 0.5, "expert_down"): 135.5e6 + 25.2e6,
                    ("cfg2", 0.5, "expert_up"): 458.2e6 + 22.1e6}
PEAK_HBM_GBS = 8000.0
N_ROTATE = 8                   # distinct x / y buffers cycled through, so that inputs come from HBM


def _time_ms(fn, steps):
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        fn(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--tau", type=float, default=0.5)
    ap.add_argument("--tokens", type=int, default=0, help="override the token count")
    ap.add_argument("--sweep", action="store_true", help="also time every tau of the workload")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 256 MiB device copy (reference for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--no-dense", action="store_true",
                    help="skip the dense-FFN comparisons (keeps a profile to the timed workload)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (tokens would shard "
              "with no exchange); run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2310_04361_amd import binding as B, cost_model, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = wl.CONFIGS[args.workload]
    if args.tokens:
        cfg = wl.with_tokens(cfg, args.tokens)
    tau = float(np.float32(args.tau))
    layer_np, x_np = wl.make_layer(cfg, 0), wl.make_input(cfg, 0)
    L = B.Layer(layer_np, cfg.dtype)
    x0 = B.to_device(x_np, cfg.dtype)
    xs = [x0] + [torch.roll(x0, shifts=17 * (i + 1), dims=0).contiguous() for i in range(N_ROTATE - 1)]
    ys = [torch.empty_like(x0) for _ in range(N_ROTATE)]
    torch.cuda.synchronize()

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # one D2D copy of 256 MiB: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    def step(i, tau=tau):
        B.dmoe_forward(L, xs[i % N_ROTATE], tau, y=ys[i % N_ROTATE])

    # executed pairs (the same for every rotated copy: the rows are only permuted)
    _, ex = B.dmoe_forward(L, x0, tau, want_lists=True)
    torch.cuda.synchronize()
    pairs = int(ex["offsets"][-1].item())
    density = pairs / (cfg.T * cfg.E)
    flops = cost_model.executed_flops(pairs, cfg.d, cfg.m, cfg.gated)

    for i in range(args.warmup):
        step(i)
    ms = _time_ms(step, args.steps)
    tokens_per_s = cfg.T / (ms * 1e-3)

    # ---- per-kernel durations (HIP events on the launch stream), separate pass
    B.timing(True)
    for i in range(min(args.steps, 200)):
        step(i)
    torch.cuda.synchronize()
    kt = {k: (n, t / n) for k, (n, t) in B.timing_read().items() if n}
    B.timing(False)
    g = 3 if cfg.gated else 2
    kflops = {"expert_up": flops * (g - 1) / g, "expert_down": flops / g}
    dom = max(kflops, key=lambda k: kt[k][1] if k in kt else 0.0)
    dom_ms = kt[dom][1]
    achieved = kflops[dom] / (dom_ms * 1e-3) / 1e12
    experts_ms = sum(kt[k][1] for k in kflops if k in kt)
    roofline = {"bound": "mfma", "kernel": dom, "achieved": round(achieved, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "traffic": MEASURED_TRAFFIC.get((cfg.name, args.tau, dom)) if not args.tokens else None,
                "avg_kernel_ms": round(dom_ms, 5),
                "experts_tflops": round(flops / (experts_ms * 1e-3) / 1e12, 2)}

    # ---- dense FFN of the same shape with the vendor GEMM (context)
    W_up = L.t["w_up"].reshape(cfg.H, cfg.d)
    W_dn = L.t["w_down"].reshape(cfg.H, cfg.d)
    W_g = L.t["w_gate"].reshape(cfg.H, cfg.d) if cfg.gated else None
    act = {"relu": torch.relu, "gelu_erf": torch.nn.functional.gelu,
           "gelu_tanh": lambda v: torch.nn.functional.gelu(v, approximate="tanh")}[cfg.act]

    def dense(i):
        x = xs[i % N_ROTATE]
        if cfg.gated:
            h = act(x @ W_g.T) * (x @ W_up.T)
        else:
            h = x @ W_up.T
            if L.t["b_up"] is not None:
                h = h + L.t["b_up"].reshape(-1)
            h = act(h)
        out = h @ W_dn
        if L.t["b_down"] is not None:
            out = out + L.t["b_down"]
        return out

    dense_ms = own_dense_ms = None
    if not args.no_dense:
        for i in range(5):
            dense(i)
        dense_ms = _time_ms(dense, 30)
        for i in range(3):
            step(i, 0.0)
        own_dense_ms = _time_ms(lambda i: step(i, 0.0), 20)

    sweep = None
    if args.sweep:
        sweep = []
        for t in cfg.taus:
            t32 = float(np.float32(t))
            _, e2 = B.dmoe_forward(L, x0, t32, want_lists=True)
            torch.cuda.synchronize()
            p = int(e2["offsets"][-1].item())
            for i in range(5):
                step(i, t32)
            m = _time_ms(lambda i: step(i, t32), 50)
            sweep.append({"tau": t, "density": round(p / (cfg.T * cfg.E), 4), "ms": round(m, 4),
                          "tokens_per_s": round(cfg.T / (m * 1e-3)),
                          "executed_tflops": round(cost_model.executed_flops(p, cfg.d, cfg.m, cfg.gated) / (m * 1e-3) / 1e12, 2),
                          "speedup_vs_dense": round(dense_ms / m, 3) if dense_ms else None})

    # ---- the oracle on the host cores, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu:
        from oracle import dmoe_oracle as oracle
        n = min(cfg.T, 16384)
        runs, t0 = 0, time.perf_counter()
        while runs < 50 and time.perf_counter() - t0 < 10.0:   # about 10 s of CPU work
            oracle.forward(layer_np, x_np[:n], tau)
            runs += 1
        dt = time.perf_counter() - t0
        cpu = {"value": round(n * runs / dt, 1), "unit": "tokens/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"first {n} tokens of {cfg.name}, tau={args.tau}, {runs} runs, {dt:.1f} s"}

    out = {
        "metric": "tokens/sec of dynamic-k MoE FFN forward (router + gate + experts)",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} d={cfg.d} E={cfg.E} m={cfg.m} d_h={cfg.d_h} "
                               f"{'gated-' if cfg.gated else ''}{cfg.act} tau={args.tau}",
                   "density": round(density, 4), "pairs": pairs},
        "executed_expert_tflops": round(flops / (ms * 1e-3) / 1e12, 2),
        "dense_ffn_ms": ({"vendor_gemm": round(dense_ms, 4), "own_kernels_tau0": round(own_dense_ms, 4)}
                         if dense_ms else None),
        "speedup_vs_dense": round(dense_ms / ms, 3) if dense_ms else None,
        "kernel_ms": {k: round(v[1], 5) for k, v in kt.items()},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    if sweep:
        out["tau_sweep"] = sweep
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
