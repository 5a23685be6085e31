#!/usr/bin/env python3
"""Benchmark of the budgeted MoE-layer forward (one step = one moespec_layer_forward call).

Workload: the OLMoE-shaped layer (d=2048, N=64, k=8, F=1024, bf16) verifying an M=63 draft tree at
budget B=32 with the substitution policy, on seeded synthetic inputs that are resident in HBM
before the timed region.  The steps cycle through several independent weight sets so that no
expert byte is served from a cache (each set is 805 MB; the last-level cache holds 256 MB).

Prints ONE JSON line: verified tree-tokens/s per MoE layer (`value`), the HBM roofline of the
dominant kernel (the gate/up pass of the expert FFN) measured with HIP events, the whole-layer
bandwidth on loaded expert bytes, a budget sweep, and the CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E bandwidth
# HBM traffic (bytes fetched + written) of one gate/up-pass launch at the default workload (olmoe_m63, B=32,
# substitution; mean over the six weight sets, 28.5 loaded experts), from the two rocprofv3 --pmc runs summarised
# in profiles/gateup_olmoe_m63_B32_hbm_traffic.md: FETCH_SIZE 117925.2 x 2.0 (copy-kernel calibration) + WRITE_SIZE
# 1011.6 KiB.  Reported only for that workload.
MEASURED_TRAFFIC_BYTES = int((117925.2 * 2.0 + 1011.6) * 1024)


def parse_args():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", default="olmoe_m63")
    ap.add_argument("--budget", type=int, default=32)
    ap.add_argument("--policy", choices=("substitution", "truncation"), default="substitution")
    ap.add_argument("--sets", type=int, default=6, help="independent weight sets cycled through (cold-cache protocol)")
    ap.add_argument("--sweep-steps", type=int, default=60)
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stream-reference", action="store_true",
                    help="skip the plain streaming read of the weights that measures the practical HBM ceiling")
    ap.add_argument("--copy-reference", action="store_true",
                    help="also run a plain 256 MiB device-to-device copy a few times: under rocprofv3 --pmc its "
                         "FETCH_SIZE / WRITE_SIZE readings calibrate the counters against a known number of bytes")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="minimum host time spent in the CPU oracle (whole layers, one weight set after another)")
    return ap.parse_args()


def make_weight_set(cfg, torch, gen, bias):
    """One independent weight set drawn on the device: N(0, sigma) rounded to bf16, shared router bias."""
    N, d, F, s = cfg.n_experts, cfg.d, cfg.d_ff, cfg.sigma_w
    def draw(*shape):
        return (torch.randn(*shape, device="cuda", generator=gen, dtype=torch.float32) * s).to(torch.bfloat16)
    return dict(w_router=draw(N, d), b_router=bias, w_gate=draw(N, F, d), w_up=draw(N, F, d), w_down=draw(N, d, F))


def timed_steps(torch, calls, steps, warmup):
    """Wall-clock ms per step of `steps` calls cycling through `calls`, synchronised on both sides."""
    R = len(calls)
    for i in range(warmup):
        calls[i % R]()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        calls[i % R]()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (no collectives, no sharding); got --gpus {args.gpus}. "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_16052_amd import binding as mb
    from paper_2602_16052_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    mb.load_library()   # fails loudly if the HIP library has not been built

    cfg = wl.CONFIGS[args.config]
    if cfg.dtype != "bf16":
        print("bench.py: the benchmark workloads are the bf16 configs", file=sys.stderr)
        sys.exit(2)
    policy = mb.SUBSTITUTE if args.policy == "substitution" else mb.TRUNCATE
    desc = mb.LayerDesc(cfg.d, cfg.n_experts, cfg.top_k, cfg.d_ff, mb.BF16, cfg.renorm)
    M, B = cfg.M, args.budget
    default_workload = (args.config, args.budget, args.policy, args.sets) == ("olmoe_m63", 32, "substitution", 6)

    gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
    bias = torch.from_numpy(wl.router_bias(cfg)).cuda()
    h = torch.randn(M, cfg.d, device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
    sets = [make_weight_set(cfg, torch, gen, bias) for _ in range(args.sets)]
    ws = mb.alloc_workspace(desc, M)
    out = torch.empty(M, cfg.d, dtype=torch.bfloat16, device="cuda")
    n_loaded_t = torch.zeros(1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()

    def loaded_experts(budget):
        counts = []
        for W in sets:
            mb.LayerForwardCall(desc, W, h, budget, policy, ws, out, n_loaded=n_loaded_t)()
            torch.cuda.synchronize()
            counts.append(int(n_loaded_t.item()))
        return sum(counts) / len(counts)

    if args.copy_reference:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- the timed region: K steps of the whole hot path, inputs resident in HBM -------------------
    calls = [mb.LayerForwardCall(desc, W, h, B, policy, ws, out) for W in sets]
    ms_per_step = timed_steps(torch, calls, args.steps, args.warmup)
    n_loaded = loaded_experts(B)
    tokens_per_s = M / (ms_per_step * 1e-3)
    layer_bytes = n_loaded * cfg.expert_bytes
    layer_gbps = layer_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- per-stage durations with HIP events recorded by the library at its stage boundaries -------
    K = min(args.steps, 200)
    traces = [mb.HipEvents(mb.TRACE_POINTS) for _ in range(K)]
    tcalls = [mb.LayerForwardCall(desc, sets[i % len(sets)], h, B, policy, ws, out, trace=traces[i]) for i in range(K)]
    for i in range(min(args.warmup, 10)):
        calls[i % len(calls)]()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for c in tcalls:
        c()
    torch.cuda.synchronize()
    ms_traced = (time.perf_counter() - t0) * 1e3 / K
    stage_ms = {name: sum(tr.elapsed_ms(i, i + 1) for tr in traces) / K for i, name in enumerate(mb.TRACE_STAGES)}
    gateup_bytes = n_loaded * 2 * cfg.d * cfg.d_ff * cfg.elem_bytes     # W_gate and W_up of every loaded expert, once
    gateup_gbps = gateup_bytes / (stage_ms["gate_up"] * 1e-3) / 1e9
    down_gbps = n_loaded * cfg.d * cfg.d_ff * cfg.elem_bytes / (stage_ms["down"] * 1e-3) / 1e9
    del tcalls, traces

    # ---- the practical ceiling: a plain streaming read of a 2 GiB buffer (8x the last-level cache), three passes ----
    stream_gbps = None
    if not args.no_stream_reference:
        big = torch.empty(2 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        cks = torch.zeros(mb.STREAM_READ_WORDS, dtype=torch.int32, device="cuda")
        mb.moespec_stream_read(big, cks)
        ev = mb.HipEvents(2)
        torch.cuda.synchronize()
        ev.record(0)
        for _ in range(3):
            mb.moespec_stream_read(big, cks)
        ev.record(1)
        torch.cuda.synchronize()
        stream_gbps = 3 * big.numel() / (ev.elapsed_ms(0, 1) * 1e-3) / 1e9
        del big

    result = {
        "metric": "verified tree-tokens/s per MoE layer",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: d={cfg.d} N={cfg.n_experts} k={cfg.top_k} F={cfg.d_ff} M={M} "
                               f"B={B} policy={args.policy} renorm={int(cfg.renorm)}",
                   "weight_sets_cycled": args.sets, "loaded_experts": n_loaded, "router_decisions": "f64"},
        "layer_hbm": {"loaded_expert_bytes": layer_bytes, "achieved_GBps": round(layer_gbps, 1),
                      "peak_GBps": HBM_PEAK_GBPS, "frac": round(layer_gbps / HBM_PEAK_GBPS, 4)},
        "roofline": {"bound": "hbm", "kernel": "expert FFN gate/up pass", "achieved": round(gateup_gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(gateup_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES if default_workload else None, "algorithmic_bytes_per_launch": gateup_bytes,
                     "avg_launch_ms": round(stage_ms["gate_up"], 5), "down_pass_GBps": round(down_gbps, 1),
                     "stream_read_GBps": round(stream_gbps, 1) if stream_gbps else None},
        "stage_ms": {k_: round(v, 5) for k_, v in stage_ms.items()},
        "ms_per_step_traced": round(ms_traced, 5),
    }

    # ---- budget sweep, including the unbudgeted (B = N) union-loading run -----------------------------
    if not args.no_sweep:
        rows = []
        budgets = sorted(set(cfg.budgets) | {cfg.n_experts})
        # quality proxies on the synthetic data (first weight set, outside the timed loops): share of the routing
        # probability held by the top-B experts, and ||O_S - O*||^2 / ||O*||^2 against the B = N output
        full, full_taps = mb.moespec_layer_forward(desc, sets[0], h, cfg.n_experts, policy, ws, taps=True)
        curve = mb.moespec_coverage_curve(desc, full_taps["scores"]).cpu().tolist()
        # the greedy oracle of Eq. (6) on the same layer: its error after B experts is the floor for any selector
        oracle_err = mb.moespec_oracle_ranking(desc, sets[0], h, cfg.n_experts, ws)[1].cpu().tolist()
        for b in budgets:
            if policy == mb.SUBSTITUTE and b < cfg.top_k:
                continue
            sc = [mb.LayerForwardCall(desc, W, h, b, policy, ws, out) for W in sets]
            ms = timed_steps(torch, sc, args.sweep_steps, 6)
            nl = loaded_experts(b)
            mb.LayerForwardCall(desc, sets[0], h, b, policy, ws, out)()
            rec = float(mb.moespec_reconstruction_error(desc, out, full, ws)[0].item())
            rows.append({"B": b, "loaded_experts": nl, "coverage": round(curve[b - 1], 4),
                         "reconstruction_error": round(rec, 5),
                         "oracle_ranking_error": round(oracle_err[b - 1], 5), "ms_per_layer": round(ms, 5),
                         "tokens_per_s": round(M / (ms * 1e-3), 1),
                         "GBps": round(nl * cfg.expert_bytes / (ms * 1e-3) / 1e9, 1),
                         "frac_of_peak": round(nl * cfg.expert_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)})
        unb = rows[-1]["ms_per_layer"]
        for r in rows:
            r["speedup_vs_unbudgeted"] = round(unb / r["ms_per_layer"], 3)
        result["sweep"] = rows

    # ---- the CPU oracle on the host cores, on a bounded sample of the same workload -------------------
    if not args.no_cpu_baseline:
        import numpy as np
        from oracle import moespec_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = 1
        pol = O.SUBSTITUTE if policy == mb.SUBSTITUTE else O.TRUNCATE
        hh = h.float().cpu().numpy()
        layers, spent = 0, 0.0
        while spent < args.cpu_seconds and layers < 64 * len(sets):
            W = sets[layers % len(sets)]
            Wh = {key: (val.float().cpu().numpy() if val.dtype == torch.bfloat16 else val.cpu().numpy())
                  for key, val in W.items()}
            t0 = time.perf_counter()
            O.layer_forward(hh, Wh, cfg.top_k, cfg.renorm, B, pol)
            spent += time.perf_counter() - t0
            layers += 1
            del Wh
        result["cpu_baseline"] = {"value": round(layers * M / spent, 3), "unit": "tokens/s", "cores": int(cores),
                                  "kind": "oracle",
                                  "sample": f"{layers} whole layers (all {M} tokens, B={B}, fp64 numpy) in {spent:.1f} s"}

    print(json.dumps(result))


if __name__ == "__main__":
    main()
