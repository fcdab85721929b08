#!/usr/bin/env python3
"""Benchmark of the dynamic-k MoE FFN forward on one MI355X.

One step = one dmoe_forward (router, gate, bucketing, experts) over one batch of synthetic
tokens that already sit in HBM.  The headline workload is the largest single-GPU configuration:
the Gemma-2B-shaped gated bf16 layer (d=2048, 256 experts of 64 neurons, gated GELU, 4096
tokens) at tau = 0.3.  Prints ONE JSON line; its "other_workloads" list carries the remaining
shapes (BERT- and ViT-shaped layers, the same gated layer at tau = 0.6 and at 16-token decode,
the attention-projection module), each with its own roofline object, and the line also holds
the speed-up-versus-density curves (tau sweep of the BERT-shaped layer, Bernoulli(p) sweep on
the shape of the paper's latency experiment) and the whole-block timing.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4] [--tau 0.3]
                    [--no-curves] [--no-others] [--no-cpu] [--no-dense]
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
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PROFILES = os.path.join(ROOT, "profiles")
N_ROTATE = 8                   # distinct x / y buffers cycled through, so that inputs come from HBM
N_LAYER_COPIES_DECODE = 4      # distinct weight copies cycled through at decode sizes: together
                               # they exceed the 256 MB last-level cache, so weights come from HBM
OTHERS = (("cfg4", 0.3), ("cfg4", 0.6), ("cfg2", 0.5), ("cfg3", 0.5), ("gemma_paper", 0.5),
          ("bert_paper", 0.5), ("cfg5a", 0.5), ("cfg5b", 0.5))


def _time_ms(fn, steps):
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        fn(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def _event_times_ms(fn, steps):
    """Per-step device time from a HIP event pair around every step on the launch stream (the
    library launches on torch's current stream): (median, min)."""
    import torch
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(steps)]
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(ev):
        a.record()
        fn(i)
        b.record()
    torch.cuda.synchronize()
    t = sorted(a.elapsed_time(b) for a, b in ev)
    return t[len(t) // 2], t[0]


def profile_traffic(name, tau, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this exact
    workload (profiles/dmoe_forward_<name>_tau<tau>_hbm_traffic.txt, lines
    `traffic <kernel> <fetch bytes> <write bytes>`), or (None, None) if there is none.  The run
    itself cannot read these counters; the file names the command that produced it."""
    path = os.path.join(PROFILES, f"dmoe_forward_{name}_tau{tau}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None, None
    with open(path) as f:
        for line in f:
            w = line.split()
            if len(w) == 4 and w[0] == "traffic" and w[1] == kernel:
                return float(w[2]) + float(w[3]), os.path.relpath(path, ROOT)
    return None, None


def achieved_peaks():
    """What this GPU delivers on the two plain limits the rooflines are quoted against: a device
    copy of 1 GiB (bytes read + written per second) and a square bf16 GEMM of 8192 (vendor
    library).  Context for the fractions of the published peaks."""
    import torch
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    copy_ms = _time_ms(lambda i: dst.copy_(src), 10)
    del src, dst
    a = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)
    b = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)
    for _ in range(2):
        a @ b
    gemm_ms = _time_ms(lambda i: a @ b, 10)
    del a, b
    torch.cuda.empty_cache()
    return {"hbm_copy_GBs": round(2 * (1 << 30) / (copy_ms * 1e-3) / 1e9, 1),
            "bf16_gemm_8192_TFLOPs": round(2 * 8192 ** 3 / (gemm_ms * 1e-3) / 1e12, 1),
            "note": "measured in this run: 1 GiB device copy (read + write), 8192^3 bf16 vendor GEMM"}


class Workload:
    """One layer + its rotated inputs on the device."""

    def __init__(self, name, tokens=0, e4m3=False, x8=False, a8=False):
        import torch
        from paper_2310_04361_amd import binding as B, workloads as wl
        cfg = wl.CONFIGS[name]
        if tokens:
            cfg = wl.with_tokens(cfg, tokens)
        self.cfg = cfg
        x8 = x8 or a8
        self.e4m3 = e4m3 or x8   # expert matrices stored in 8-bit E4M3 (one byte per weight)
        self.layer_np, self.x_np = wl.make_layer(cfg, 0), wl.make_input(cfg, 0)
        if e4m3 or x8:
            self.layer_np = wl.quantize_experts_e4m3(self.layer_np)
        if x8:   # ... and the experts' input quantised row-wise to E4M3 as well
            self.layer_np["x8"] = True
        if a8:   # ... and every row of hidden activations too
            self.layer_np["a8"] = True
        self.decode = cfg.T <= 16
        n_layers = N_LAYER_COPIES_DECODE if self.decode else 1
        self.layers = [B.Layer(self.layer_np, cfg.dtype) for _ in range(n_layers)]
        x0 = B.to_device(self.x_np, cfg.dtype)
        self.xs = [x0] + [torch.roll(x0, shifts=17 * (i + 1), dims=0).contiguous()
                          for i in range(N_ROTATE - 1)]
        self.ys = [torch.empty_like(x0) for _ in range(N_ROTATE)]
        torch.cuda.synchronize()

    def step(self, i, tau, hot=False):
        from paper_2310_04361_amd import binding as B
        L = self.layers[0 if hot else i % len(self.layers)]
        B.dmoe_forward(L, self.xs[i % N_ROTATE], tau, y=self.ys[i % N_ROTATE])

    def measure(self, tau_arg, steps, warmup, traffic_ok=True):
        """Whole-forward time, per-kernel times (HIP events stamped by the launches themselves) and the
        roofline object of the dominant expert kernel."""
        import torch
        from paper_2310_04361_amd import binding as B, cost_model
        cfg = self.cfg
        tau = float(np.float32(tau_arg))
        # executed pairs (the same for every rotated copy: the rows are only permuted)
        _, ex = B.dmoe_forward(self.layers[0], self.xs[0], tau, want_lists=True)
        torch.cuda.synchronize()
        offsets = ex["offsets"].cpu().numpy()
        pairs = int(offsets[-1])
        touched = int(np.count_nonzero(np.diff(offsets)))
        flops = cost_model.executed_flops(pairs, cfg.d, cfg.m, cfg.gated)

        for i in range(warmup):
            self.step(i, tau)
        ms = _time_ms(lambda i: self.step(i, tau), steps)
        ev_median, ev_min = _event_times_ms(lambda i: self.step(i, tau), min(steps, 200))

        B.timing(True)
        for i in range(min(steps, 200)):
            self.step(i, tau)
        torch.cuda.synchronize()
        kt = {k: t / n for k, (n, t) in B.timing_read().items() if n}
        B.timing(False)

        g = 3 if cfg.gated else 2
        if self.decode:
            # weight-streaming kernels: algorithmic bytes = the touched experts' weights, once
            per_expert = (1.0 if self.e4m3 else 2.0) * cfg.d * cfg.m
            kbytes = {"small_up": touched * per_expert * (g - 1), "small_down": touched * per_expert}
            dom = max(kbytes, key=lambda k: kt.get(k, 0.0))
            achieved = kbytes[dom] / (kt[dom] * 1e-3) / 1e9
            both_ms = kt["small_up"] + kt["small_down"]
            traffic, source = profile_traffic(cfg.name, tau_arg, dom) if (traffic_ok and not self.e4m3) else (None, None)
            roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1),
                        "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBS, 4),
                        "traffic": traffic, "traffic_source": source, "avg_kernel_ms": round(kt[dom], 5),
                        "touched_experts": touched,
                        "experts_gbs": round(sum(kbytes.values()) / (both_ms * 1e-3) / 1e9, 1),
                        "weight_copies_rotated": len(self.layers)}
        else:
            # two down kernels are launched; the one the density selects does the work
            down = max(("expert_down", "expert_down_sparse"), key=lambda k: kt.get(k, 0.0))
            kflops = {"expert_up": flops * (g - 1) / g, down: flops / g}
            dom = max(kflops, key=lambda k: kt.get(k, 0.0))
            achieved = kflops[dom] / (kt[dom] * 1e-3) / 1e12
            # (layers with 8-bit inputs run their up-projection on the fp8 matrix pipe, whose peak
            # is twice this one: their line is context, the bf16 layers are the roofline claim)
            experts_ms = sum(kt.get(k, 0.0) for k in ("expert_up", "expert_down", "expert_down_sparse"))
            traffic, source = profile_traffic(cfg.name, tau_arg, dom) if (traffic_ok and not self.e4m3) else (None, None)
            roofline = {"bound": "mfma", "kernel": dom, "achieved": round(achieved, 2),
                        "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                        "traffic": traffic, "traffic_source": source,
                        "avg_kernel_ms": round(kt[dom], 5),
                        "experts_tflops": round(flops / (experts_ms * 1e-3) / 1e12, 2),
                        "experts_frac": round(flops / (experts_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
        return {"ms": ms, "ms_event_median": ev_median, "ms_event_min": ev_min, "pairs": pairs,
                "density": pairs / (cfg.T * cfg.E), "flops": flops,
                "kernel_ms": {k: round(v, 5) for k, v in kt.items()}, "roofline": roofline}

    def dense_ms(self):
        """Dense FFN of the same shape with the vendor GEMM (context)."""
        import torch
        cfg, L = self.cfg, self.layers[0]
        W_up = L.t["w_up"].reshape(cfg.H, cfg.d)
        W_dn = L.t["w_down"].reshape(cfg.H, cfg.d)
        W_g = L.t["w_gate"].reshape(cfg.H, cfg.d) if cfg.gated else None
        act = {"relu": torch.relu, "gelu_erf": torch.nn.functional.gelu,
               "gelu_tanh": lambda v: torch.nn.functional.gelu(v, approximate="tanh")}[cfg.act]

        def dense(i):
            x = self.xs[i % N_ROTATE]
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

        for i in range(5):
            dense(i)
        return _time_ms(dense, 30)

    def describe(self, tau):
        cfg = self.cfg
        return (f"{cfg.name}: T={cfg.T} d={cfg.d} E={cfg.E} m={cfg.m} d_h={cfg.d_h} "
                f"{'gated-' if cfg.gated else ''}{cfg.act} tau={tau}")


def encoder_block_timing(tau_arg=0.5, heads=12):
    """ViT-B-shaped pre-norm encoder block on the 256x197-token tensor of the paper's latency
    experiment: x + Attn(LN(x)), then + FFN(LN(.)).  Everything but the FFN is vendor code (torch
    LayerNorm, GEMMs, scaled-dot-product attention) and only serves as the fixed part of the
    block; the FFN is either the dense vendor-GEMM FFN or dmoe_forward on the ViT-shaped layer
    (cfg3).  The FFN input is the cfg3 tensor itself, so that the density is the one reported for
    cfg3; the two parts are timed in sequence on one stream but their data are not chained."""
    import torch
    import torch.nn.functional as F
    from paper_2310_04361_amd import binding as B
    w = Workload("cfg3")
    cfg, L = w.cfg, w.layers[0]
    tau = float(np.float32(tau_arg))
    Bt, S, d = 256, 197, cfg.d
    g = torch.Generator(device="cuda").manual_seed(0)
    wqkv = (torch.randn(3 * d, d, device="cuda", generator=g) / d ** 0.5).to(torch.bfloat16)
    wo = (torch.randn(d, d, device="cuda", generator=g) / d ** 0.5).to(torch.bfloat16)
    ln_w = torch.ones(d, device="cuda", dtype=torch.bfloat16)
    ln_b = torch.zeros(d, device="cuda", dtype=torch.bfloat16)
    W_up, W_dn = L.t["w_up"].reshape(cfg.H, d), L.t["w_down"].reshape(cfg.H, d)

    def attention_part(i):
        x = w.xs[i % N_ROTATE]
        hdn = F.layer_norm(x, (d,), ln_w, ln_b)
        qkv = (hdn @ wqkv.T).view(Bt, S, 3, heads, d // heads).permute(2, 0, 3, 1, 4)
        a = F.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2])
        a = a.transpose(1, 2).reshape(Bt * S, d) @ wo.T
        y1 = x + a
        return y1, F.layer_norm(y1, (d,), ln_w, ln_b)

    def dense_ffn(i):
        x = w.xs[i % N_ROTATE]
        hdn = F.gelu(x @ W_up.T + L.t["b_up"].reshape(-1))
        return hdn @ W_dn + L.t["b_down"]

    def block_dense(i):
        y1, _ = attention_part(i)
        return y1 + dense_ffn(i)

    def block_dmoe(i):
        y1, _ = attention_part(i)
        B.dmoe_forward(L, w.xs[i % N_ROTATE], tau, y=w.ys[i % N_ROTATE])
        return y1 + w.ys[i % N_ROTATE]

    res = {}
    for name, fn in (("attention_part_ms", attention_part), ("dense_ffn_ms", dense_ffn),
                     ("dmoe_ffn_ms", lambda i: w.step(i, tau)),
                     ("block_dense_ms", block_dense), ("block_dmoe_ms", block_dmoe)):
        for i in range(3):
            fn(i)
        res[name] = round(_time_ms(fn, 20), 4)
    res["ffn_speedup"] = round(res["dense_ffn_ms"] / res["dmoe_ffn_ms"], 3)
    res["block_speedup"] = round(res["block_dense_ms"] / res["block_dmoe_ms"], 3)
    res["workload"] = f"ViT-B-shaped block, {Bt}x{S} tokens, d={d}, {heads} heads; FFN = {w.describe(tau_arg)}"
    res["note"] = ("LayerNorm, projections and attention are vendor (torch) kernels; only the FFN "
                   "differs between the two block timings")
    del w
    torch.cuda.empty_cache()
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg4")
    ap.add_argument("--tau", type=float, default=0.3)
    ap.add_argument("--tokens", type=int, default=0, help="override the token count")
    ap.add_argument("--sweep", action="store_true", help="also time every tau of the headline workload")
    ap.add_argument("--no-curves", action="store_true",
                    help="skip the speed-up-versus-density curves (tau sweep of the BERT-shaped layer, "
                         "Bernoulli(p) sweep on the shape of Sec. 4.4) and the whole-block timing")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-others", action="store_true", help="skip the other workloads")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 256 MiB device copy (reference for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--top-k", type=int, default=0,
                    help="also time the headline workload with the top-k gate (k experts per token)")
    ap.add_argument("--paper-sweep", action="store_true",
                    help="(default unless --no-curves) time dmoe_expert_ffn on the paper's benchmark "
                         "shape (24 experts x 128, d=768, 256x197 tokens) under Bernoulli(p) "
                         "decisions, p = 0 .. 1 (Sec. 4.4)")
    ap.add_argument("--block", action="store_true",
                    help="(default unless --no-curves) time a ViT-B-shaped encoder block (LayerNorm, "
                         "12-head attention, residuals, FFN) on 256x197 tokens with the dense FFN and "
                         "with the dynamic-k layer in its place (Sec. 4.4: what survives end to end)")
    ap.add_argument("--x8", action="store_true",
                    help="with --no-others: still time the headline layer with 8-bit weights and inputs")
    ap.add_argument("--a8", action="store_true",
                    help="with --no-others: still time the headline layer fully 8-bit (hidden activations too)")
    ap.add_argument("--no-dense", action="store_true",
                    help="skip the dense-FFN comparisons (keeps a profile to the timed workload)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (tokens would shard "
              "with no exchange); run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2310_04361_amd import binding as B, cost_model

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = Workload(args.workload, args.tokens)
    cfg = w.cfg
    tau = float(np.float32(args.tau))

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # one D2D copy of 256 MiB: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    r = w.measure(args.tau, args.steps, args.warmup, traffic_ok=not args.tokens)
    ms = r["ms"]

    dense_ms = own_dense_ms = None
    if not args.no_dense:
        dense_ms = w.dense_ms()
        for i in range(3):
            w.step(i, 0.0)
        own_dense_ms = _time_ms(lambda i: w.step(i, 0.0), 20)

    def tau_sweep(wl_, dms):
        rows = []
        c = wl_.cfg
        for t in c.taus:
            t32 = float(np.float32(t))
            _, e2 = B.dmoe_forward(wl_.layers[0], wl_.xs[0], t32, want_lists=True)
            torch.cuda.synchronize()
            p = int(e2["offsets"][-1].item())
            for i in range(5):
                wl_.step(i, t32)
            m = _time_ms(lambda i: wl_.step(i, t32), 50)
            rows.append({"tau": t, "density": round(p / (c.T * c.E), 4), "ms": round(m, 4),
                         "tokens_per_s": round(c.T / (m * 1e-3)),
                         "executed_tflops": round(cost_model.executed_flops(p, c.d, c.m, c.gated) / (m * 1e-3) / 1e12, 2),
                         "speedup_vs_dense": round(dms / m, 3) if dms else None})
        return rows

    def measure_other(wo, name, t, dms):
        steps = 100 if wo.cfg.T > 16 else 400
        ro = wo.measure(t, steps, 10)
        entry = {"workload": wo.describe(t), "ms_per_step": round(ro["ms"], 5),
                 "ms_per_step_event_median": round(ro["ms_event_median"], 5),
                 "ms_per_step_event_min": round(ro["ms_event_min"], 5),
                 "tokens_per_s": round(wo.cfg.T / (ro["ms"] * 1e-3), 1),
                 "density": round(ro["density"], 4), "pairs": ro["pairs"],
                 "executed_expert_tflops": round(ro["flops"] / (ro["ms"] * 1e-3) / 1e12, 2),
                 "dense_vendor_gemm_ms": round(dms, 4) if dms else None,
                 "speedup_vs_dense": round(dms / ro["ms"], 3) if dms else None,
                 "kernel_ms": ro["kernel_ms"], "roofline": ro["roofline"]}
        if wo.decode:
            t32 = float(np.float32(t))
            hot = _time_ms(lambda i: wo.step(i, t32, hot=True), steps)
            entry["ms_per_step_weights_cached"] = round(hot, 5)
            # the same forward recorded once per weight copy as a HIP graph and replayed
            graphs = []
            for li, Lc in enumerate(wo.layers):
                gph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gph):
                    B.dmoe_forward(Lc, wo.xs[li], t32, y=wo.ys[li])
                graphs.append(gph)
            for gph in graphs:
                gph.replay()
            entry["ms_per_step_graph_replay"] = round(
                _time_ms(lambda i: graphs[i % len(graphs)].replay(), steps), 5)
            del graphs
            if name == "cfg5b":
                # the query / key / value modules of one attention layer (Sec. 3.5): three
                # layers of this shape on one input, one launch per stage for the group
                qkv = wo.layers[:3]
                ys3 = [torch.empty_like(wo.ys[0]) for _ in range(3)]
                taus3 = [t32] * 3
                for i in range(5):
                    B.dmoe_forward_group(qkv, wo.xs[i % N_ROTATE], taus3, ys=ys3)
                grp = _time_ms(lambda i: B.dmoe_forward_group(qkv, wo.xs[i % N_ROTATE], taus3, ys=ys3), steps)

                def three(i):
                    for li in range(3):
                        B.dmoe_forward(qkv[li], wo.xs[i % N_ROTATE], t32, y=ys3[li])
                sep = _time_ms(three, steps)
                gph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gph):
                    B.dmoe_forward_group(qkv, wo.xs[0], taus3, ys=ys3)
                gph.replay()
                rep = _time_ms(lambda i: gph.replay(), steps)
                entry["qkv_group"] = {"layers": 3, "ms_group_call": round(grp, 5),
                                      "ms_three_single_calls": round(sep, 5),
                                      "ms_group_graph_replay": round(rep, 5)}
                del gph
        return entry

    sweep = tau_sweep(w, dense_ms) if args.sweep else None

    # ---- the oracle on the host cores, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu:
        from oracle import dmoe_oracle as oracle
        # about 10 s of CPU work: a sample of at most 16384 tokens, fewer for the wide gated layer
        # whose tokens cost ten times as much
        n = min(cfg.T, 16384 if cfg.d * cfg.m * (3 if cfg.gated else 2) < 100000 else 1024)
        runs, t0 = 0, time.perf_counter()
        while runs < 50 and time.perf_counter() - t0 < 10.0:
            oracle.forward(w.layer_np, w.x_np[:n], tau)
            runs += 1
        dt = time.perf_counter() - t0
        cpu = {"value": round(n * runs / dt, 1), "unit": "tokens/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"first {n} tokens of {cfg.name}, tau={args.tau}, {runs} runs, {dt:.1f} s"}

    out = {
        "metric": "tokens/sec of dynamic-k MoE FFN forward (router + gate + experts)",
        "value": round(cfg.T / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": w.describe(args.tau), "density": round(r["density"], 4),
                   "pairs": r["pairs"]},
        "ms_per_step_event_median": round(r["ms_event_median"], 5),
        "ms_per_step_event_min": round(r["ms_event_min"], 5),
        "executed_expert_tflops": round(r["flops"] / (ms * 1e-3) / 1e12, 2),
        "executed_expert_frac_of_mfma_peak": round(r["flops"] / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "dense_ffn_ms": ({"vendor_gemm": round(dense_ms, 4), "own_kernels_tau0": round(own_dense_ms, 4)}
                         if dense_ms else None),
        "speedup_vs_dense": round(dense_ms / ms, 3) if dense_ms else None,
        "kernel_ms": r["kernel_ms"],
        "roofline": r["roofline"],
        "cpu_baseline": cpu,
        "achieved_peak": achieved_peaks(),
    }
    if sweep:
        out["tau_sweep"] = sweep

    # the same forward recorded as HIP graphs (one per rotated input) and replayed: what a caller
    # that captures the layer pays, without the launch gaps between its six kernels
    graphs = []
    for gi in range(N_ROTATE):
        gph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gph):
            B.dmoe_forward(w.layers[0], w.xs[gi], tau, y=w.ys[gi])
        graphs.append(gph)
    for gph in graphs:
        gph.replay()
    out["ms_per_step_graph_replay"] = round(_time_ms(lambda i: graphs[i % N_ROTATE].replay(), args.steps), 5)
    del graphs

    if args.top_k:
        k = args.top_k
        for i in range(5):
            B.dmoe_forward_topk(w.layers[0], w.xs[i % N_ROTATE], k, y=w.ys[i % N_ROTATE])
        m = _time_ms(lambda i: B.dmoe_forward_topk(w.layers[0], w.xs[i % N_ROTATE], k,
                                                   y=w.ys[i % N_ROTATE]), 100)
        out["top_k_gate"] = {"k": k, "ms_per_step": round(m, 5),
                             "tokens_per_s": round(cfg.T / (m * 1e-3), 1),
                             "speedup_vs_dense": round(dense_ms / m, 3) if dense_ms else None}

    # the headline layer at its other thresholds, while it is on the device
    others, done_names = [], set()
    if not args.no_others and not args.tokens:
        for name, t in OTHERS:
            if name == args.workload and t != args.tau:
                others.append(measure_other(w, name, t, dense_ms))
        done_names.add(args.workload)
    del w
    torch.cuda.empty_cache()

    if (not args.no_others or args.x8 or args.a8) and not args.tokens and cfg.dtype == "bf16":
        # the same layer with 8-bit expert weights and 8-bit (row-wise E4M3) expert inputs: the
        # up-projection of wide experts runs on the fp8 matrix pipe (Appendix C's lower precisions)
        same_layer = [] if args.no_others else [o for o in OTHERS if o[0] == args.workload and o[1] != args.tau]
        for key, kw, note in [
                ("fp8_inputs_and_weights", {"x8": True},
                 "weight_format DMOE_W_FP8_E4M3_X8 (8-bit expert weights and inputs, bf16 hidden "
                 "activations): same shapes, a different (lower) precision -- not the bf16 headline"),
                ("fp8_fully_8bit", {"a8": True},
                 "weight_format DMOE_W_FP8_E4M3_A8 (8-bit expert weights, inputs and hidden "
                 "activations: both expert products on the fp8 matrix pipe): same shapes, a "
                 "different (lower) precision -- not the bf16 headline")]:
            if args.no_others and not (args.a8 if "a8" in kw else args.x8):
                continue
            w8 = Workload(args.workload, **kw)
            rows = []
            for name, t in [(args.workload, args.tau)] + same_layer:
                r8 = w8.measure(t, 100, 10)
                rows.append({"workload": w8.describe(t), "ms_per_step": round(r8["ms"], 5),
                             "executed_expert_tflops": round(r8["flops"] / (r8["ms"] * 1e-3) / 1e12, 2),
                             "kernel_ms": r8["kernel_ms"]})
            out[key] = {"note": note, "rows": rows}
            del w8
            torch.cuda.empty_cache()

    curves = not args.no_curves
    if curves and not args.tokens:
        # speed-up against density on the BERT-shaped layer (tau = 0.1 .. 0.9)
        w2 = Workload("cfg2")
        d2 = None if args.no_dense else w2.dense_ms()
        out["cfg2_tau_sweep"] = {"workload": w2.describe("0.1..0.9"),
                                 "dense_vendor_gemm_ms": round(d2, 4) if d2 else None,
                                 "rows": tau_sweep(w2, d2)}
        del w2
        torch.cuda.empty_cache()

    if args.paper_sweep or curves:
        from paper_2310_04361_amd import workloads as wl
        pw = Workload("paper")
        pw8 = Workload("paper", a8=True)   # the same layer fully 8-bit (Appendix C's precision table)
        pc, pL, pL8 = pw.cfg, pw.layers[0], pw8.layers[0]
        pd = None if args.no_dense else pw.dense_ms()
        rows = []
        for p in (0.0, 0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9, 1.0):
            mask = wl.bernoulli_mask(pc.T, pc.E, p, seed=7)
            offs = np.concatenate([[0], np.cumsum(mask.sum(axis=0))]).astype(np.int32)
            lists = np.concatenate([np.flatnonzero(mask[:, e]) for e in range(pc.E)] + [np.zeros(1)]).astype(np.int32)
            offs_d, lists_d = torch.from_numpy(offs).cuda(), torch.from_numpy(lists).cuda()
            ms = []
            for lay, w in ((pL, pw), (pL8, pw8)):
                for i in range(3):
                    B.dmoe_expert_ffn(lay, w.xs[i % N_ROTATE], offs_d, lists_d)
                ms.append(_time_ms(lambda i: B.dmoe_expert_ffn(lay, w.xs[i % N_ROTATE], offs_d, lists_d), 20))
            rows.append({"p": p, "ms": round(ms[0], 4), "ms_fully_8bit": round(ms[1], 4),
                         "vs_dense": round(pd / ms[0], 3) if pd else None})
        out["paper_shape_bernoulli_sweep"] = {"workload": pw.describe("-"), "note": "dmoe_expert_ffn "
                                              "only (decisions given, no router), as in Sec. 4.4; "
                                              "ms: bf16 layer, ms_fully_8bit: weight format "
                                              "DMOE_W_FP8_E4M3_A8 (the precisions of Appendix C's table)",
                                              "dense_vendor_gemm_ms": round(pd, 4) if pd else None,
                                              "rows": rows}
        del pw, pw8

    if args.block or curves:
        out["encoder_block"] = encoder_block_timing()

    if not args.no_others:
        for name, t in OTHERS:
            if (name, t) == (args.workload, args.tau) or name in done_names:
                continue
            wo = Workload(name)
            dms = None if args.no_dense else wo.dense_ms()
            for name2, t2 in OTHERS:
                if name2 == name:
                    others.append(measure_other(wo, name, t2, dms))
            done_names.add(name)
            if name == "cfg5a":
                # the same layer with its expert matrices stored in 8-bit E4M3: half the weight
                # bytes per touched expert
                del wo
                torch.cuda.empty_cache()
                w8 = Workload(name, e4m3=True)
                r8 = w8.measure(t, 400, 10)
                others[-1]["e4m3_weights"] = {"ms_per_step": round(r8["ms"], 5),
                                              "kernel_ms": r8["kernel_ms"], "roofline": r8["roofline"]}
                del w8
            wo = None
            torch.cuda.empty_cache()
        out["other_workloads"] = others
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
