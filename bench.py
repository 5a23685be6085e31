#!/usr/bin/env python3
"""Benchmark of the budgeted MoE-layer forward (one step = one moespec_layer_forward call: all steps of the hot path).

Headline workload: the OLMoE-shaped layer (d=2048, N=64, k=8, F=1024, bf16) verifying an M=63 draft tree at budget
B=32 with the substitution policy.  The inputs are the seeded synthetic tensors of paper_2602_16052_amd/workloads.py
(seeds 0..5: six independent layers, 805 MB of experts each), resident in HBM before the timed region; the steps
cycle through the six layers so that no expert byte is served from a cache (the last-level cache holds 256 MB).
Before anything is timed, the layer of seed 0 is checked against the CPU oracle (routing ids exact, every token's
output within tolerance); a mismatch ends the run with a non-zero status.

Prints ONE JSON line: verified tree-tokens/s per MoE layer (`value`), whole-layer bandwidth on loaded expert bytes
(`layer_hbm`), the HBM roofline of the dominant kernel (gate/up pass of the expert FFN, HIP-event timing inside this
run), a budget sweep with the unbudgeted B=N run, the other workloads (larger trees, 128 experts, the 8-layer coarse
stack) each with its own sweep, and the CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E bandwidth
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "gateup_olmoe_m63_B32_hbm_traffic.md")
TRACE_PROFILE = os.path.join(ROOT, "profiles", "bench_olmoe_m63_B32_kernel_trace.md")
TOL_BF16 = 2e-2


def parse_args():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", default="olmoe_m63")
    ap.add_argument("--budget", type=int, default=32)
    ap.add_argument("--policy", choices=("substitution", "truncation"), default="substitution")
    ap.add_argument("--sets", type=int, default=6, help="independent seeded layers cycled through (cold-cache protocol)")
    ap.add_argument("--sweep-steps", type=int, default=60)
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-workloads", action="store_true", help="skip the other workloads (larger trees, 128 experts, stack)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stream-reference", action="store_true",
                    help="skip the plain streaming read that measures the practical HBM ceiling")
    ap.add_argument("--copy-reference", action="store_true",
                    help="also run a plain 256 MiB device-to-device copy a few times: under rocprofv3 --pmc its "
                         "FETCH_SIZE / WRITE_SIZE readings calibrate the counters against a known number of bytes")
    ap.add_argument("--cpu-seconds", type=float, default=10.0,
                    help="host time spent in the CPU oracle with all BLAS threads (a third of it again single-threaded)")
    return ap.parse_args()


def source_hash() -> str:
    """sha256 over the kernel sources: ties a stored profile to the build it was measured on."""
    hsh = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2602_16052_amd", "csrc", "*"))):
        with open(path, "rb") as f:
            hsh.update(os.path.basename(path).encode() + b"\0" + f.read())
    return hsh.hexdigest()[:16]


def stored_traffic():
    """(bytes per gate/up launch, note) from the tracked rocprofv3 counter summary, if it was measured on this build."""
    try:
        text = open(TRAFFIC_PROFILE).read()
        sha = re.search(r"csrc_sha256_16:\s*([0-9a-f]{16})", text).group(1)
        val = int(re.search(r"traffic_bytes_per_launch:\s*(\d+)", text).group(1))
    except (OSError, AttributeError):
        return None, "no counter summary under profiles/"
    if sha != source_hash():
        return None, f"counter summary under profiles/ was measured on another build ({sha})"
    return val, "FETCH_SIZE + WRITE_SIZE of profiles/" + os.path.basename(TRAFFIC_PROFILE)


def stored_kernel_trace():
    """Average gate/up kernel duration (ms) of the tracked rocprofv3 kernel-trace summary, if measured on this build."""
    try:
        text = open(TRACE_PROFILE).read()
        sha = re.search(r"csrc_sha256_16:\s*([0-9a-f]{16})", text).group(1)
        us = float(re.search(r"gateup_kernel_trace_avg_us:\s*([0-9.]+)", text).group(1))
    except (OSError, AttributeError):
        return None
    return us * 1e-3 if sha == source_hash() else None


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


def stack_main(args, cfg, policy, torch, np, mb, wl, O):
    """--config coarse_stack: one step = moespec_stack_forward over the 8 layers (every pass reads 22.5 GB of distinct
    experts, so every pass is cold); figures are per layer, t_stack / n_layers."""
    desc = mb.LayerDesc(cfg.d, cfg.n_experts, cfg.top_k, cfg.d_ff, mb.BF16, cfg.renorm)
    gen = torch.Generator(device="cuda").manual_seed(1234)
    rnd = lambda *shape: (torch.randn(*shape, device="cuda", generator=gen, dtype=torch.float32) * cfg.sigma_w).to(torch.bfloat16)
    layers = [dict(w_router=rnd(cfg.n_experts, cfg.d), b_router=torch.from_numpy(wl.router_bias(cfg, layer=l)).cuda(),
                   w_gate=rnd(cfg.n_experts, cfg.d_ff, cfg.d), w_up=rnd(cfg.n_experts, cfg.d_ff, cfg.d),
                   w_down=rnd(cfg.n_experts, cfg.d, cfg.d_ff)) for l in range(cfg.n_layers)]
    h0 = torch.randn(cfg.M, cfg.d, device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
    ws = mb.alloc_workspace(desc, cfg.M)
    B = args.budget if args.budget <= cfg.n_experts else 4
    tok = torch.empty((cfg.n_layers, cfg.M, cfg.top_k), dtype=torch.int32, device="cuda")
    h_run = h0.clone()
    call = mb.StackForwardCall(desc, layers, h_run, B, policy, ws, pre_norm=True, tok_ids=tok)
    steps, warmup = min(args.steps, 50), min(args.warmup, 5)
    for _ in range(max(warmup, 1)):
        h_run.copy_(h0)
        call()
    torch.cuda.synchronize()
    nl = float(np.mean([len(set(tok[l].flatten().tolist()) - {-1}) for l in range(cfg.n_layers)]))
    spent = 0.0
    for _ in range(steps):          # the hidden state is reset outside the timed interval of every pass
        h_run.copy_(h0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        call()
        torch.cuda.synchronize()
        spent += time.perf_counter() - t0
    ms_layer = spent * 1e3 / steps / cfg.n_layers
    gbps = nl * cfg.expert_bytes / (ms_layer * 1e-3) / 1e9
    print(json.dumps({
        "metric": "verified tree-tokens/s per MoE layer", "value": round(cfg.M / (ms_layer * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_layer * cfg.n_layers, 5),
        "ms_per_layer": round(ms_layer, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_layers} layers, d={cfg.d} N={cfg.n_experts} k={cfg.top_k} F={cfg.d_ff} "
                               f"M={cfg.M} B={B} policy={args.policy}, h <- h + MoE_S(rms_scale(h)); one step = one "
                               "moespec_stack_forward over all layers", "loaded_experts": nl,
                   "inputs": "drawn on the device (torch), same distributions as workloads.py"},
        "layer_hbm": {"loaded_expert_bytes": nl * cfg.expert_bytes, "achieved_GBps": round(gbps, 1),
                      "peak_GBps": HBM_PEAK_GBPS, "frac": round(gbps / HBM_PEAK_GBPS, 4)}}))


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (no collectives, no sharding); got --gpus {args.gpus}. "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_16052_amd import binding as mb
    from paper_2602_16052_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    mb.load_library()   # fails loudly if the HIP library has not been built
    from oracle import moespec_oracle as O   # the parity gate and the cpu_baseline leg only

    cfg = wl.CONFIGS[args.config]
    if cfg.dtype != "bf16":
        print("bench.py: the benchmark workloads are the bf16 configs", file=sys.stderr)
        sys.exit(2)
    policy = mb.SUBSTITUTE if args.policy == "substitution" else mb.TRUNCATE
    if cfg.n_layers > 1:
        stack_main(args, cfg, policy, torch, np, mb, wl, O)
        return
    o_policy = O.SUBSTITUTE if policy == mb.SUBSTITUTE else O.TRUNCATE
    M, B = cfg.M, args.budget

    def to_device(x):
        if x.dtype == np.uint16:
            return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(x).cuda()

    def desc_of(c):
        return mb.LayerDesc(c.d, c.n_experts, c.top_k, c.d_ff, mb.BF16, c.renorm,
                            mb.GATE_SIGMOID if c.gate == "sigmoid" else mb.GATE_SOFTMAX)

    desc = desc_of(cfg)

    # ---- seeded inputs: layer `i` of the cycle is the workload drawn from seed cfg.seed + i ------------------------
    host0 = None
    sets = []
    for i in range(args.sets):
        W = wl.layer_weights(cfg, seed=cfg.seed + i, threads=16)
        h = wl.hidden_states(cfg, seed=cfg.seed + i)
        if i == 0:
            host0 = (W, h)
        sets.append(({key: to_device(val) for key, val in W.items()}, to_device(h)))
    ws = mb.alloc_workspace(desc, M)
    out = torch.empty(M, cfg.d, dtype=torch.bfloat16, device="cuda")
    n_loaded_t = torch.zeros(1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()

    def oracle_check(c, d_, W_dev, h_dev, budget, pol, o_pol, tokens=None, W_host=None):
        """Routing of every token and the outputs of `tokens` (None: all) of one GPU layer call against the oracle."""
        out_g, taps = mb.moespec_layer_forward(d_, W_dev, h_dev, budget, pol, mb.alloc_workspace(d_, h_dev.shape[0]), taps=True)
        torch.cuda.synchronize()
        f32 = lambda t: t.float().cpu().numpy()
        h_o = f32(h_dev)
        g, ids, w = O.route(h_o, f32(W_dev["w_router"]), W_dev["b_router"].cpu().numpy(), c.top_k, c.renorm, c.gate)
        ref = O.budget(g, ids, w, budget, o_pol, c.top_k, c.renorm)
        ids_exact = bool(np.array_equal(taps["budget_ids"].cpu().numpy()[:budget], ref["S"]) and
                         np.array_equal(taps["tok_ids"].cpu().numpy(), ref["tok_ids"]) and
                         np.array_equal(taps["perm"].cpu().numpy()[:int(ref["seg_off"][-1])], ref["perm"]))
        rows = list(range(h_dev.shape[0])) if tokens is None else list(tokens)
        need = sorted({int(e) for t in rows for e in ref["tok_ids"][t] if e >= 0})
        Wexp = {key: {e: f32(W_dev[key][e]) for e in need} for key in ("w_gate", "w_up", "w_down")}
        want = O.combine(h_o, ref["tok_ids"], ref["tok_w"], Wexp["w_gate"], Wexp["w_up"], Wexp["w_down"], tokens=rows)
        got = out_g.float().cpu().numpy().astype(np.float64)
        err = float(np.max(np.abs(got[rows] - want[rows])))
        scale = float(np.max(np.abs(want[rows])))
        ok = ids_exact and err <= TOL_BF16 * max(1.0, scale) and bool(np.all(np.isfinite(got)))
        return {"ids_exact": ids_exact, "max_abs": round(err, 6), "max_abs_oracle": round(scale, 4),
                "tokens_compared": len(rows), "tolerance": TOL_BF16, "ok": ok}

    # ---- parity gate on the tensors that are about to be timed (layer of seed 0, every token) ----------------------
    parity = oracle_check(cfg, desc, sets[0][0], sets[0][1], B, policy, o_policy)
    if not parity["ok"]:
        print(json.dumps({"error": "GPU layer differs from the CPU oracle on the benchmark's own inputs", "parity": parity}))
        sys.exit(3)

    def loaded_experts(d_, the_sets, budget, pol, ws_, out_):
        counts = []
        for W, h in the_sets:
            mb.LayerForwardCall(d_, W, h, budget, pol, ws_, out_, n_loaded=n_loaded_t)()
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

    # ---- the timed region: K steps of the whole hot path, inputs resident in HBM -----------------------------------
    calls = [mb.LayerForwardCall(desc, W, h, B, policy, ws, out) for W, h in sets]
    # the GPU has idled while the host drew the inputs: bring its clocks back up before the W warm-up steps (with few
    # of those, e.g. 5, the first timed steps would otherwise run on a GPU still ramping up: +5 us per step at K=20)
    for i in range(240):
        calls[i % len(calls)]()
    torch.cuda.synchronize()
    ms_per_step = timed_steps(torch, calls, args.steps, args.warmup)
    n_loaded = loaded_experts(desc, sets, B, policy, ws, out)
    tokens_per_s = M / (ms_per_step * 1e-3)
    layer_bytes = n_loaded * cfg.expert_bytes
    layer_gbps = layer_bytes / (ms_per_step * 1e-3) / 1e9

    def stage_times(d_, the_sets, budget, pol, ws_, out_, K):
        """Average stage durations (ms) from HIP events the library records at its stage boundaries."""
        traces = [mb.HipEvents(mb.TRACE_POINTS) for _ in range(K)]
        tcalls = [mb.LayerForwardCall(d_, the_sets[i % len(the_sets)][0], the_sets[i % len(the_sets)][1], budget, pol, ws_,
                                      out_, trace=traces[i]) for i in range(K)]
        for i in range(min(10, K)):
            mb.LayerForwardCall(d_, the_sets[i % len(the_sets)][0], the_sets[i % len(the_sets)][1], budget, pol, ws_, out_)()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for c in tcalls:
            c()
        torch.cuda.synchronize()
        ms_traced = (time.perf_counter() - t0) * 1e3 / K
        st = {name: sum(tr.elapsed_ms(i, i + 1) for tr in traces) / K for i, name in enumerate(mb.TRACE_STAGES)}
        return st, ms_traced

    stage_ms, ms_traced = stage_times(desc, sets, B, policy, ws, out, min(args.steps, 200))
    gateup_bytes = n_loaded * 2 * cfg.d * cfg.d_ff * cfg.elem_bytes     # W_gate and W_up of every loaded expert, once
    gateup_gbps = gateup_bytes / (stage_ms["gate_up"] * 1e-3) / 1e9
    down_gbps = n_loaded * cfg.d * cfg.d_ff * cfg.elem_bytes / (stage_ms["down"] * 1e-3) / 1e9

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

    # what an event interval carries besides the kernel: two records with nothing between them, on an idle stream
    ev = mb.HipEvents(2)
    empty = []
    for _ in range(50):
        ev.record(0)
        ev.record(1)
        torch.cuda.synchronize()
        empty.append(ev.elapsed_ms(0, 1))
    event_overhead_ms = sorted(empty)[len(empty) // 2]

    default_workload = (args.config, args.budget, args.policy, args.sets) == ("olmoe_m63", 32, "substitution", 6)
    traffic, traffic_note = stored_traffic() if default_workload else (None, "measured for the default workload only")
    trace_ms = stored_kernel_trace() if default_workload else None
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
                   "inputs": f"workloads.py seeds {cfg.seed}..{cfg.seed + args.sets - 1}, one layer per seed, cycled",
                   "weight_sets_cycled": args.sets, "loaded_experts": n_loaded, "router_decisions": "f64"},
        "parity": parity,
        "layer_hbm": {"loaded_expert_bytes": layer_bytes, "achieved_GBps": round(layer_gbps, 1),
                      "peak_GBps": HBM_PEAK_GBPS, "frac": round(layer_gbps / HBM_PEAK_GBPS, 4)},
        "roofline": {"bound": "hbm", "kernel": "expert FFN gate/up pass", "achieved": round(gateup_gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(gateup_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": traffic, "traffic_source": traffic_note, "build": source_hash(),
                     "algorithmic_bytes_per_launch": gateup_bytes,
                     "avg_launch_ms": round(stage_ms["gate_up"], 5),
                     "empty_event_interval_ms": round(event_overhead_ms, 5),
                     "kernel_trace_avg_launch_ms": round(trace_ms, 5) if trace_ms else None,
                     "kernel_trace_frac": round(gateup_bytes / trace_ms / 1e6 / HBM_PEAK_GBPS, 4) if trace_ms else None,
                     "down_pass_GBps": round(down_gbps, 1),
                     "stream_read_GBps": round(stream_gbps, 1) if stream_gbps else None},
        "stage_ms": {k_: round(v, 5) for k_, v in stage_ms.items()},
        "ms_per_step_traced": round(ms_traced, 5),
    }

    def sweep_rows(c, d_, the_sets, budgets, pol, ws_, out_, steps, quality=False):
        """One row per budget: time per layer, loaded experts, bandwidth on loaded bytes; speedup over B = N."""
        rows = []
        full = curve = oracle_err = None
        if quality:
            # quality proxies on the synthetic data (first layer of the cycle, outside the timed loops): share of the
            # routing probability held by the top-B experts, ||O_S - O*||^2 / ||O*||^2 against the B = N output, and
            # the same for the greedy oracle ranking of Eq. (6), the floor for any selector
            full, full_taps = mb.moespec_layer_forward(d_, the_sets[0][0], the_sets[0][1], c.n_experts, pol, ws_, taps=True)
            curve = mb.moespec_coverage_curve(d_, full_taps["scores"]).cpu().tolist()
            oracle_err = mb.moespec_oracle_ranking(d_, the_sets[0][0], the_sets[0][1], c.n_experts, ws_)[1].cpu().tolist()
        for b in budgets:
            if pol == mb.SUBSTITUTE and b < c.top_k:
                continue
            sc = [mb.LayerForwardCall(d_, W, h, b, pol, ws_, out_) for W, h in the_sets]
            ms = timed_steps(torch, sc, steps, 6)
            nl = loaded_experts(d_, the_sets, b, pol, ws_, out_)
            gbps = nl * c.expert_bytes / (ms * 1e-3) / 1e9
            row = {"B": b, "loaded_experts": round(nl, 2), "ms_per_layer": round(ms, 5),
                   "tokens_per_s": round(c.M / (ms * 1e-3), 1), "GBps": round(gbps, 1),
                   "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4)}
            if quality:
                mb.LayerForwardCall(d_, the_sets[0][0], the_sets[0][1], b, pol, ws_, out_)()
                rec = float(mb.moespec_reconstruction_error(d_, out_, full, ws_)[0].item())
                row.update(coverage=round(curve[b - 1], 4), reconstruction_error=round(rec, 5),
                           oracle_ranking_error=round(oracle_err[b - 1], 5))
            rows.append(row)
        unb = rows[-1]["ms_per_layer"]
        for r in rows:
            r["speedup_vs_unbudgeted"] = round(unb / r["ms_per_layer"], 3)
        return rows

    # ---- budget sweep of the headline workload, including the unbudgeted (B = N) union-loading run ------------------
    if not args.no_sweep:
        result["sweep"] = sweep_rows(cfg, desc, sets, sorted(set(cfg.budgets) | {cfg.n_experts}), policy, ws, out,
                                     args.sweep_steps, quality=True)

    # ---- the CPU oracle on the host cores, on a bounded sample of the same workload ----------------------------------
    if not args.no_cpu_baseline:
        W0, h0 = host0
        Wh = {key: wl.as_f32(val) for key, val in W0.items()}
        hh = wl.as_f32(h0)

        def oracle_rate(seconds):
            layers, spent = 0, 0.0
            while spent < seconds and layers < 256:
                t0 = time.perf_counter()
                O.layer_forward(hh, Wh, cfg.top_k, cfg.renorm, B, o_policy)
                spent += time.perf_counter() - t0
                layers += 1
            return layers, spent

        try:
            from threadpoolctl import threadpool_info, threadpool_limits
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threadpool_limits, cores = None, 1
        layers, spent = oracle_rate(args.cpu_seconds)
        base = {"value": round(layers * M / spent, 3), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
                "sample": f"{layers} whole layers of seed {cfg.seed} (all {M} tokens, B={B}, fp64 numpy with its BLAS "
                          f"threads; not the optimisation target) in {spent:.1f} s"}
        if threadpool_limits is not None:
            with threadpool_limits(limits=1):
                l1, s1 = oracle_rate(args.cpu_seconds / 3)
            base["single_thread"] = {"value": round(l1 * M / s1, 3), "unit": "tokens/s", "cores": 1,
                                     "sample": f"{l1} whole layers in {s1:.1f} s"}
        result["cpu_baseline"] = base
        del Wh
    del calls, sets, host0
    torch.cuda.empty_cache()

    # ---- the other workloads: larger trees, the 128-expert shape, the 8-layer coarse stack ---------------------------
    if not args.no_workloads:
        gen = torch.Generator(device="cuda").manual_seed(1234)

        def draw_layer(c, layer_seed):
            """One layer drawn on the device: N(0, sigma) rounded to bf16, the workload's seeded router bias."""
            N_, d_, F_, s_ = c.n_experts, c.d, c.d_ff, c.sigma_w
            rnd = lambda *shape: (torch.randn(*shape, device="cuda", generator=gen, dtype=torch.float32) * s_).to(torch.bfloat16)
            return dict(w_router=rnd(N_, d_), b_router=torch.from_numpy(wl.router_bias(c, layer=layer_seed)).cuda(),
                        w_gate=rnd(N_, F_, d_), w_up=rnd(N_, F_, d_), w_down=rnd(N_, d_, F_))

        others = []
        shared = {}   # the three OLMoE-shaped trees share their weight sets; only the hidden rows differ
        for name, n_sets in (("olmoe_m127", 4), ("fine_m127", 3), ("olmoe_m255", 4), ("olmoe_m511", 4)):
            c = wl.CONFIGS[name]
            d_ = desc_of(c)
            key = (c.d, c.n_experts, c.d_ff, c.bias_alpha)
            if key not in shared:
                shared.clear()
                torch.cuda.empty_cache()
                shared[key] = [draw_layer(c, i) for i in range(n_sets)]
            the_sets = [(W, torch.randn(c.M, c.d, device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16))
                        for W in shared[key]]
            ws_ = mb.alloc_workspace(d_, c.M)
            out_ = torch.empty(c.M, c.d, dtype=torch.bfloat16, device="cuda")
            head_B = 32 if 32 in c.budgets else c.budgets[0]
            rows = sweep_rows(c, d_, the_sets, sorted(set(c.budgets) | {c.n_experts}), policy, ws_, out_, 30)
            st, _ = stage_times(d_, the_sets, head_B, policy, ws_, out_, 40)
            sample = sorted({int(t) for t in np.linspace(0, c.M - 1, 4)})
            others.append({"workload": f"{c.name}: d={c.d} N={c.n_experts} k={c.top_k} F={c.d_ff} M={c.M} "
                                       f"policy={args.policy}", "inputs": f"drawn on the device (torch, {n_sets} layers "
                           "cycled), same distributions as workloads.py", "sweep": rows,
                           "stage_ms_at_B%d" % head_B: {k_: round(v, 5) for k_, v in st.items()},
                           "parity_at_B%d" % head_B: oracle_check(c, d_, the_sets[0][0], the_sets[0][1], head_B, policy,
                                                                  o_policy, tokens=sample)})
            del the_sets, ws_, out_
        shared.clear()
        torch.cuda.empty_cache()

        # the stack: one step = moespec_stack_forward over its 8 layers (22.5 GB of experts: every pass is cold);
        # reported per layer as t_stack / 8
        c = wl.CONFIGS["coarse_stack"]
        d_ = desc_of(c)
        layers = [draw_layer(c, l) for l in range(c.n_layers)]
        h0 = torch.randn(c.M, c.d, device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
        ws_ = mb.alloc_workspace(d_, c.M)
        rows = []
        for b in c.budgets:
            tok = torch.empty((c.n_layers, c.M, c.top_k), dtype=torch.int32, device="cuda")
            h_run = h0.clone()
            call = mb.StackForwardCall(d_, layers, h_run, b, policy, ws_, pre_norm=True, tok_ids=tok)
            call()
            torch.cuda.synchronize()
            nl = float(np.mean([len(set(tok[l].flatten().tolist()) - {-1}) for l in range(c.n_layers)]))
            steps = 6
            times = []
            for _ in range(steps):      # the hidden state is reset outside the timed interval of every pass
                h_run.copy_(h0)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                call()
                torch.cuda.synchronize()
                times.append((time.perf_counter() - t0) * 1e3)
            ms = sorted(times)[len(times) // 2] / c.n_layers
            gbps = nl * c.expert_bytes / (ms * 1e-3) / 1e9
            rows.append({"B": b, "loaded_experts": round(nl, 2), "ms_per_layer": round(ms, 5),
                         "ms_per_stack": round(ms * c.n_layers, 4), "tokens_per_s": round(c.M / (ms * 1e-3), 1),
                         "GBps": round(gbps, 1), "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4)})
        unb = rows[-1]["ms_per_layer"]
        for r in rows:
            r["speedup_vs_unbudgeted"] = round(unb / r["ms_per_layer"], 3)
        x0 = mb.moespec_rms_scale(d_, h0)
        others.append({"workload": f"{c.name}: {c.n_layers} layers, d={c.d} N={c.n_experts} k={c.top_k} F={c.d_ff} "
                                   f"M={c.M} policy={args.policy}, h <- h + MoE_S(rms_scale(h))",
                       "inputs": "drawn on the device (torch), same distributions as workloads.py; one step = "
                                 "moespec_stack_forward over the 8 layers, ms_per_layer = t_stack / 8 (median of 6 passes)",
                       "sweep": rows,
                       "parity_layer0_at_B4": oracle_check(c, d_, layers[0], x0, 4, policy, o_policy, tokens=[0, 31, 62])})
        result["workloads"] = others

    print(json.dumps(result))


if __name__ == "__main__":
    main()
