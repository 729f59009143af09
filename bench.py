#!/usr/bin/env python3
"""Prefill throughput of libpo on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: every request
of the workload goes through po_prefill (embedding -> L x [norm, QKV, RoPE, attention over
the whole sequence, O-proj, norm, chunked SwiGLU MLP] -> last-row norm + LM head -> label
log-probs).  Default workload: the Llama-3-8B-shaped bf16 model on one 32768-token request,
MLP chunk 4096 (the configuration the headline metric is quoted on).

Prints ONE JSON line (see the keys below).  `value` is tokens/s with weights and workspace
resident in HBM; the only host traffic inside the timed region is the 128 KiB of token ids
going in and the logits coming out.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import numpy as np

PEAK_BF16_TFLOPS = 2516.6      # MI355X dense bf16 MFMA: 256 CU x 2.4 GHz x 4096 flop/clk/CU
PEAK_FP8_TFLOPS = 5033.2       # dense fp8 MFMA: twice the bf16 rate
PEAK_HBM_GBS = 8000.0

def load_traffic(workload):
    """Measured HBM-side traffic per launch of each kernel class, from the committed summary of two rocprofv3
    counter runs of this command (FETCH_SIZE, then WRITE_SIZE; profiles/prefill_<workload>_pmc_counters.txt, written
    by paper_2505_07203_amd/pmc_summary.py).  The summary records a hash of the kernel sources it measured; it is
    used only if the sources are unchanged, else every traffic is null.
    -> ({class: bytes per launch}, file name) or ({}, None)"""
    from paper_2505_07203_amd import pmc_summary
    path = os.path.join(ROOT, "profiles", f"prefill_{workload}_pmc_counters.txt")
    if not os.path.exists(path):
        return {}, None
    out, sha = {}, None
    with open(path) as f:
        for line in f:
            part = line.rstrip("\n").split("\t")
            if part[0] == "traffic_bytes_per_launch" and len(part) >= 4:
                out[part[1]] = float(part[3])
            elif part[0] == "kernel_sources_sha256" and len(part) >= 2:
                sha = part[1]
    if not out or sha != pmc_summary.kernel_sources_sha256():
        return {}, None                               # measured on other kernels than today's: stale
    return out, os.path.relpath(path, ROOT)


def flop_model(cfg, lens, lazy_last_layer=True):
    """Algorithmic flops: causal half of attention only, LM head on the last row only and, with the
    last-layer shortcut the library runs by default, the last layer's query projection, attention,
    O-projection and MLP for the last position only (no credit for work that is not needed: the
    kernels still compute the whole 256-row block of that position)."""
    per_class = flop_classes(cfg, lens, lazy_last_layer)
    return per_class["qkv"] + per_class["residual"] + per_class["gate_up"] + per_class["lm_head"], per_class["attention"]


def flop_classes(cfg, lens, lazy_last_layer=True):
    d, F, qd, kvd, L = cfg.d_model, cfg.ffn_dim, cfg.q_dim, cfg.kv_dim, cfg.n_layers
    out = dict.fromkeys(("qkv", "residual", "gate_up", "attention", "lm_head"), 0.0)
    for n in lens:
        n = float(n)
        full = L - 1 if lazy_last_layer else L          # layers that run on every position
        out["qkv"] += full * 2.0 * d * (qd + 2 * kvd) * n
        out["residual"] += full * 2.0 * (qd * d + F * d) * n
        out["gate_up"] += full * 2.0 * d * 2 * F * n
        out["attention"] += full * 4.0 * qd * n * (n + 1) / 2
        if lazy_last_layer:                             # last layer: K, V everywhere; the rest for one row
            out["qkv"] += 2.0 * d * 2 * kvd * n + 2.0 * d * qd
            out["residual"] += 2.0 * (qd * d + F * d)
            out["gate_up"] += 2.0 * d * 2 * F
            out["attention"] += 4.0 * qd * n
        out["lm_head"] += 2.0 * d * cfg.vocab_size
    return out


def cpu_baseline(cfg, wseed, tseed, full_lens, sample_layers, sample_tokens):
    """Times the oracle as it stands on a bounded slice of the same workload (first
    `sample_layers` layers x first `sample_tokens` tokens) and scales by the flop model."""
    from oracle import prefill_oracle as O
    import helpers as H
    from paper_2505_07203_amd import inputs as I
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    scfg = cfg.replace(n_layers=sample_layers)
    tokens = I.make_tokens(cfg, tseed, sample_tokens)
    # only the embedding rows the sample reads are widened to fp64 (same values, less memory)
    embed = I.stored_to_f64(I.make_tensor(cfg, wseed, I.KIND_EMBED, -1)[tokens])
    layers = [H.oracle_layer(cfg, wseed, l) for l in range(sample_layers)]
    t0 = time.perf_counter()
    O.forward_hidden(np.arange(sample_tokens), embed, layers, scfg)
    dt = time.perf_counter() - t0
    lin_s, att_s = flop_model(scfg, [sample_tokens], lazy_last_layer=False)   # the oracle slice runs every row
    lin_s -= 2.0 * cfg.d_model * cfg.vocab_size          # the slice stops before the LM head
    lin_f, att_f = flop_model(cfg, full_lens)
    full_time = dt * (lin_f + att_f) / (lin_s + att_s)
    return {"value": float(sum(full_lens)) / full_time, "unit": "tokens/s", "cores": int(cores),
            "kind": "oracle",
            "sample": f"fp64 numpy oracle, first {sample_layers} layer(s) x first {sample_tokens} tokens of the "
                      f"same workload: {dt:.2f} s measured, extrapolated to the full workload by the flop model"}


def cpu_baseline_full_tiny():
    """The oracle timed IN FULL on the small fp32 configuration (2 layers, 512 tokens), nothing extrapolated."""
    from oracle import prefill_oracle as O   # noqa: F401  (imported by helpers below; named here for the reader)
    import helpers as H
    from paper_2505_07203_amd import inputs as I
    w = I.WORKLOADS["tiny_512"]
    tokens = I.make_tokens(w["cfg"], w["tseed"], w["lens"][0])
    t0 = time.perf_counter()
    H.oracle_prefill(w["cfg"], w["wseed"], tokens, cand=I.label_ids(w["cfg"]))
    dt = time.perf_counter() - t0
    return {"workload": "tiny_512", "value": w["lens"][0] / dt, "unit": "tokens/s", "seconds": dt, "kind": "oracle",
            "sample": "the whole configuration (weights generated inside the timed region)"}


def cpu_baseline_full_request():
    """The oracle timed IN FULL on the shortest request of the 16-request mix (all 32 layers at the 8B width): minutes
    of CPU time, so only on request (--cpu-baseline-request)."""
    import helpers as H
    from paper_2505_07203_amd import inputs as I
    w = I.WORKLOADS["llama8b_mixed16"]
    lens = [int(n) for n in I.workload_lengths("llama8b_mixed16")]
    i = min(range(len(lens)), key=lambda j: lens[j])
    tokens = I.make_tokens(w["cfg"], w["tseed"], int(lens[i]), request=i)
    t0 = time.perf_counter()
    H.oracle_prefill(w["cfg"], w["wseed"], tokens, cand=I.label_ids(w["cfg"]))
    dt = time.perf_counter() - t0
    return {"workload": "llama8b_mixed16", "request": i, "tokens": lens[i], "value": lens[i] / dt, "unit": "tokens/s",
            "seconds": dt, "kind": "oracle", "sample": "one whole request, all layers (weights generated inside the timed region)"}


def cpu_baseline_recorded():
    """What tests/golden/make_golden.py recorded when it ran the oracle over the WHOLE 16-request mix (all layers, exact
    mode): read from the fixture, not measured now, and on that machine's cores."""
    path = os.path.join(ROOT, "tests", "golden", "llama8b_mixed16.json")
    try:
        with open(path) as f:
            g = json.load(f)
        toks = sum(r["len"] for r in g["requests"])
        return {"workload": "llama8b_mixed16", "tokens": toks, "value": toks / g["oracle_layer_seconds_exact_mode"],
                "unit": "tokens/s", "seconds": g["oracle_layer_seconds_exact_mode"], "cores": g.get("host_cores"),
                "kind": "oracle, recorded", "sample": "all 16 requests x 32 layers, layer time of the exact evaluation as "
                "recorded in tests/golden/llama8b_mixed16.json when the fixture was written"}
    except (OSError, KeyError, ValueError):
        return None


def micro_peaks(B, torch):
    """Measured micro-peaks beside the nominal ones: matrix-instruction loops on random bf16 operands (no memory
    traffic inside the loop; the rate is what the board's power limit grants) and a 1 GiB streaming copy."""
    out = {}
    n_op = 1024 * 512 * 32
    operands = (torch.randn(n_op // 2, device="cuda") * 0.5).to(torch.bfloat16)
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for name, kind, wps in (("mfma_32x32x16_bf16_1_wave_per_simd", 0, 1), ("mfma_32x32x16_bf16_2_waves_per_simd", 0, 2),
                            ("mfma_16x16x32_bf16_1_wave_per_simd", 1, 1), ("mfma_16x16x32_bf16_2_waves_per_simd", 1, 2)):
        B.po_op_mfma_peak(kind, wps, 2000, operands, sink)               # warm-up, also brings the clock down
        torch.cuda.synchronize()
        e0.record()
        flop = B.po_op_mfma_peak(kind, wps, 20000 if kind else 40000, operands, sink)
        e1.record()
        torch.cuda.synchronize()
        out[name + "_tflops"] = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    B.po_op_stream_copy(src, dst)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(10):
        B.po_op_stream_copy(src, dst)
    e1.record()
    torch.cuda.synchronize()
    out["stream_copy_gbs_read_plus_write"] = 10 * 2 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9
    out["nominal"] = {"bf16_mfma_tflops": PEAK_BF16_TFLOPS, "hbm_gbs": PEAK_HBM_GBS}
    return out


def footprint_sweep(B, I, cfg, chunk, main_ctx, main_len):
    """Peak HBM against input length: the closed form (po_workspace_bytes) for 4 k .. 128 k tokens beside the
    model of an engine that keeps every layer's K/V and does not chunk the MLP, and the profile run's measured
    high-water mark at three lengths (the main context's, and one-layer contexts for the others: the activation
    arena does not depend on the layer count)."""
    d, F, L = cfg.d_model, cfg.ffn_dim, cfg.n_layers
    naive_slope = 2 * (L * 2 * cfg.kv_dim + 4 * d + 3 * F)      # bytes per token: all-layer K/V + X, Xn, Q, O + GU + H
    rows = []
    for n in (4096, 8192, 16384, 32768, 65536, 131072):
        wb, sb = B.po_workspace_bytes(cfg, n, chunk)
        rows.append({"tokens": n, "weights_bytes": wb, "workspace_bytes": sb, "naive_activation_bytes": naive_slope * n})
    measured = []
    for n in (4096, main_len, 131072):
        if n == main_len:
            _, touched = main_ctx.po_profile(n)
            measured.append({"tokens": n, "layers": cfg.n_layers, "touched_bytes": touched, "closed_form_bytes": main_ctx.workspace_bytes})
            continue
        c1 = cfg.replace(n_layers=1)
        ctx = B.Context(c1, n, chunk)
        try:
            ctx.load_synthetic(1, threads=16)
            _, touched = ctx.po_profile(n)
            measured.append({"tokens": n, "layers": 1, "touched_bytes": touched, "closed_form_bytes": ctx.workspace_bytes})
        finally:
            ctx.po_destroy()
    return {"mlp_chunk": chunk, "closed_form": rows, "profile_run": measured,
            "bytes_per_token": {"this_path": (rows[-1]["workspace_bytes"] - rows[-2]["workspace_bytes"]) / 65536.0,
                                "all_layer_kv_unchunked_mlp": naive_slope}}


def sample_shader_clock(run_step, n_steps=2):
    """Shader clock (MHz, rocm-smi) and package power (W, the driver's hwmon sensor) while `run_step` keeps the GPU busy;
    outside the timed region.  -> (median clock, {median power, power cap}), each None when its source is not there."""
    import re
    import subprocess
    import threading
    import glob
    clocks, watts, stop = [], [], threading.Event()
    hwmon = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input")[:1]

    def poll():
        while not stop.is_set():
            try:
                r = subprocess.run(["/opt/rocm/bin/rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=5)
                for line in r.stdout.splitlines():
                    m = re.search(r"sclk clock level.*\((\d+)Mhz\)", line)
                    if m:
                        clocks.append(int(m.group(1)))
                for f in hwmon:                 # (the driver's own sensor file, microwatts; rocm-smi prints no power here)
                    with open(f) as fh:
                        watts.append(float(fh.read().strip()) / 1e6)
            except Exception:
                return
            time.sleep(0.15)
    th = threading.Thread(target=poll, daemon=True)
    th.start()
    for _ in range(n_steps):
        run_step()
    stop.set()
    th.join(timeout=10)

    def median_busy(v):
        busy = sorted(v[1:]) if len(v) > 2 else sorted(v)
        return busy[len(busy) // 2] if busy else None
    cap = None
    for f in glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_cap")[:1]:
        try:
            with open(f) as fh:
                cap = float(fh.read().strip()) / 1e6
        except Exception:
            pass
    return median_busy(clocks), {"during_untimed_steps": median_busy(watts), "cap": cap}


def serve(args, cfg, w, B, I):
    """Section 7's evaluation loop on one GPU with synthetic requests: users arrive (all at once, or as a
    Poisson process), each with all of its requests; every step the engine takes one waiting request.  The
    service times are real (wall clock around po_engine_step, host scheduling included), the arrival
    clock is simulated: it advances by each step's duration, or jumps to the next arrival when idle."""
    import numpy as np
    trace = I.make_serving_trace(cfg, args.serve, w["tseed"], args.serve_users, args.serve_posts)
    users = [u for u, _ in trace]
    n_users = len(set(users))
    max_len = max(len(t) for _, t in trace)
    cand = I.label_ids(cfg)
    ctx = B.Context(cfg, max_len, w["chunk"])
    ctx.load_synthetic(w["wseed"], threads=16)
    ctx.po_set_few_rows_split(not args.serve_default_path)
    cache_bytes = 0

    def drain(lam, user_arrival, request_arrival=None):
        nonlocal cache_bytes
        cache_bytes = ctx.po_attach_kv_cache(max_len, n_slots=args.serve_slots)     # a fresh, empty cache
        sch = B.Scheduler(lam)
        # requests of one arrival instant keep the trace's order: a nanosecond apart
        arr = [user_arrival[u] + 1e-9 * i for i, u in enumerate(users)]
        if args.serve_interleave:
            # round robin over users: post k of every user before post k + 1 of any; with a rate, one request per
            # arrival of the Poisson process instead of one user
            seen, rank = {}, []
            for u in users:
                rank.append(seen.get(u, 0))
                seen[u] = rank[-1] + 1
            order = sorted(range(len(users)), key=lambda i: (rank[i], users[i]))
            times = request_arrival if request_arrival is not None else [0.0] * len(users)
            for pos, i in enumerate(order):
                arr[i] = times[pos] + 1e-9 * pos
        todo = sorted(range(len(trace)), key=lambda i: arr[i])
        now, k, done, busy, hits, tokens, computed = 0.0, 0, {}, 0.0, 0, 0, 0
        while k < len(todo) or sch.po_sched_size():
            while k < len(todo) and arr[todo[k]] <= now:
                sch.po_sched_push(todo[k], trace[todo[k]][1], arr[todo[k]])
                k += 1
            if not sch.po_sched_size():
                now = arr[todo[k]]
                continue
            t0 = time.perf_counter()
            rid, n, reused, _, _ = ctx.po_engine_step(sch, now, cand)
            dt = time.perf_counter() - t0
            now += dt
            busy += dt
            done[rid] = now - arr[rid]
            hits += reused > 0
            tokens += n
            computed += n - reused
        lat = np.asarray([done[i] for i in range(len(trace))])
        return {"requests_per_s": len(trace) / busy, "tokens_per_s": tokens / busy, "computed_tokens_per_s": computed / busy,
                "busy_s": busy, "makespan_s": now, "mean_latency_s": float(lat.mean()), "p99_latency_s": float(np.percentile(lat, 99)),
                "requests_that_reused_a_prefix": int(hits)}

    x = drain(500.0, [0.0] * n_users)["requests_per_s"]                             # warm-up; sets the rate unit
    rows = []
    for rate in [float(r) for r in args.serve_rates.split(",")]:
        ra = None
        if rate == 0:
            ua = [0.0] * n_users
        else:
            ua = I.poisson_user_arrivals(w["tseed"], n_users, rate * x * n_users / len(trace)).tolist()
            if args.serve_interleave:
                ra = I.poisson_user_arrivals(w["tseed"], len(trace), rate * x).tolist()
        # (arrival order = lambda so large that a nanosecond of queuing outweighs any JCT)
        for policy, lam in (("arrival_order", 1e18), ("srjf_calibrated_lambda500", 500.0)):
            r = drain(lam, ua, ra)
            r.update(policy=policy, arrival="all_at_once" if rate == 0 else f"poisson_{rate:g}x")
            rows.append(r)
    ctx.po_destroy()
    best = max(r["requests_per_s"] for r in rows)
    print(json.dumps({"metric": "prefill_only_serving_requests_per_s", "value": best, "unit": "requests/s", "n_gpus": 1,
                      "higher_is_better": True, "dtype": "fp8_e4m3 linear layers, bf16 elsewhere" if args.fp8 else "bf16",
                      "data": "synthetic", "vs_baseline": None,
                      "config": {"workload": f"{args.serve} trace on the {args.workload} model shape", "users": n_users,
                                 "requests": len(trace), "max_request_tokens": max_len,
                                 "total_tokens": int(sum(len(t) for _, t in trace)),
                                 "prefix_cache_entries": args.serve_slots, "prefix_cache_bytes": int(cache_bytes),
                                 "few_rows_split": not args.serve_default_path, "interleaved_arrivals": bool(args.serve_interleave)},
                      "runs": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="llama8b_32k")
    ap.add_argument("--layers", type=int, default=0, help="debug: override the layer count (invalidates the metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-request", action="store_true",
                    help="also time the oracle in full on the shortest request of the 16-request mix (minutes of CPU time)")
    ap.add_argument("--no-phase-timing", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the untimed extras: micro-peaks (matrix loop, streaming copy) and the footprint sweep")
    ap.add_argument("--no-clock-sample", action="store_true",
                    help="skip the two extra, untimed steps during which the shader clock is read from rocm-smi")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one elementwise kernel that reads 1 GiB and writes 1 GiB, so that a "
                         "counter run of this command holds a dispatch of known HBM traffic")
    ap.add_argument("--reuse-prefix", type=int, default=0,
                    help="also time the first request again with the K/V of its first P tokens in the prefix "
                         "cache (reported under prefix_reuse; not part of value)")
    ap.add_argument("--jct-profile", type=int, default=0, metavar="STEP",
                    help="also profile the request time over (n_input, n_cached) pairs at this granularity in tokens "
                         "(the paper uses 1000), fit the scheduler's linear model and report how well the number of "
                         "cache-miss tokens tracks the time (reported under jct_profile; not part of value)")
    ap.add_argument("--serve", default="", choices=["", "postrec", "credit"],
                    help="instead of the prefill metric: drain a synthetic serving trace with the structure of one of the "
                         "paper's two evaluation workloads through po_engine_step (scheduler + prefix cache + prefill), "
                         "arrival order against the calibrated schedule; prints its own JSON line")
    ap.add_argument("--serve-users", type=int, default=0, help="override the trace's number of users")
    ap.add_argument("--serve-posts", type=int, default=0, help="override the trace's requests per user")
    ap.add_argument("--serve-slots", type=int, default=4, help="entries of the prefix cache")
    ap.add_argument("--serve-interleave", action="store_true",
                    help="the requests of different users arrive interleaved (round robin over users, one request at a "
                         "time) instead of user by user: arrival order then loses the cached prefixes (Section 6.2)")
    ap.add_argument("--serve-default-path", action="store_true",
                    help="serve on the default (bit-reproducible across row sets) path instead of few-rows mode")
    ap.add_argument("--serve-rates", default="0,1",
                    help="arrival rates to run, as multiples of the drain throughput measured with everything "
                         "arriving at once (0 = all at once); users arrive as a Poisson process")
    ap.add_argument("--fp8", action="store_true",
                    help="variant: the decoder's linear layers run FP8-dynamic (E4M3 weights per output channel, "
                         "activations per token); reported under its own metric name and dtype, never as the bf16 metric")
    ap.add_argument("--few-rows", action="store_true",
                    help="variant: few-rows mode (po_set_few_rows_split) for launches with few rows; reported in config")
    ap.add_argument("--packed", type=int, default=0,
                    help="variant: run the workload's requests through po_prefill_packed with buffers of this many "
                         "rows (consecutive short requests share the launches of the position-wise layers)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (requests are independent; more GPUs run more "
              "independent engine instances); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2505_07203_amd import binding as B
    from paper_2505_07203_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    w = I.WORKLOADS[args.workload]
    cfg = w["cfg"]
    if args.layers:
        cfg = cfg.replace(n_layers=args.layers)
    if args.fp8:
        cfg = cfg.replace(dtype=I.BF16_FP8)
    if args.serve:
        serve(args, cfg, w, B, I)
        return
    lens = [int(x) for x in I.workload_lengths(args.workload)]
    cand = I.label_ids(cfg)
    reqs = [I.make_tokens(cfg, w["tseed"], n, request=i) for i, n in enumerate(lens)]

    t0 = time.perf_counter()
    ctx = B.Context(cfg, max(max(lens), args.packed), w["chunk"])
    ctx.load_synthetic(w["wseed"], threads=16)
    load_s = time.perf_counter() - t0
    ctx.po_set_phase_timing(False)
    ctx.po_set_few_rows_split(args.few_rows)

    classes = B.KERNEL_CLASSES

    def step():
        ms = dict.fromkeys(classes, 0.0)
        n = dict.fromkeys(classes, 0)
        for t in ([None] if args.packed else reqs):
            if args.packed:
                ctx.po_prefill_packed(reqs, cand)
            else:
                ctx.po_prefill(t, cand, want_logits=len(reqs) == 1)
            st = ctx.po_get_stats()
            for k in classes:
                ms[k] += st["kernel_ms"][k]
                n[k] += st["kernel_launches"][k]
        return ms, n

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        B.po_op_stream_copy(src, dst)         # 2^30 bytes fetched, 2^30 bytes written
        torch.cuda.synchronize()
        del src, dst
    # ---- pass 1, the metric: K steps with nothing but the path on the stream (no per-launch events)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    # ---- pass 2, the per-kernel split: the same steps again with a HIP event pair around every attention and
    # GEMM launch, recorded on the path's stream (about 900 pairs per step; this pass is not part of `value`)
    k_ms = dict.fromkeys(classes, 0.0)
    k_n = dict.fromkeys(classes, 0)
    split_steps = 0
    ms_per_step_with_events = None
    if not args.no_phase_timing:
        ctx.po_set_phase_timing(True)
        step()
        torch.cuda.synchronize()
        split_steps = max(1, min(args.steps, 5))
        t1 = time.perf_counter()
        for _ in range(split_steps):
            ms, n = step()
            for k in classes:
                k_ms[k] += ms[k]
                k_n[k] += n[k]
        torch.cuda.synchronize()
        ms_per_step_with_events = 1e3 * (time.perf_counter() - t1) / split_steps
        ctx.po_set_phase_timing(False)
    sclk, watts = (None, {"during_untimed_steps": None, "cap": None}) if args.no_clock_sample else sample_shader_clock(step)
    tokens = sum(lens)
    value = tokens * args.steps / elapsed
    lin_f, att_f = flop_model(cfg, lens)
    chunk = w["chunk"]
    free_b, total_b = torch.cuda.mem_get_info()
    # algorithmic flops per step of each kernel class (causal half only for attention)
    k_flop = flop_classes(cfg, lens)
    gk = "gemm_fp8_mfma_kernel" if args.fp8 else "gemm_bf16_mfma_kernel"
    k_name = {"attention": ("attn_fwd64_kernel" if cfg.head_dim == 128 else "attn_fwd_kernel<64>") +
                           " (causal GQA flash attention, one launch per layer)",
              "qkv": gk + "<3> (QKV projection + RoPE + transposed V)",
              "residual": gk + "<1> (O-projection and MLP down projection + residual)",
              "gate_up": gk + "<2> (MLP gate/up projection + SiLU-multiply)"}

    traffic, traffic_file = ({}, None) if (args.layers or args.fp8 or args.packed or args.few_rows) else load_traffic(args.workload)

    def roof(k):
        launches = k_n[k] / max(split_steps, 1)
        avg_ms = k_ms[k] / max(k_n[k], 1)
        ach = k_flop[k] / max(launches, 1) / 1e12 / (avg_ms / 1e3) if avg_ms > 0 else 0.0
        peak = PEAK_FP8_TFLOPS if (args.fp8 and k != "attention") else PEAK_BF16_TFLOPS
        return {"kernel": k_name[k], "bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                "frac": ach / peak, "traffic": traffic.get(k), "traffic_source": traffic_file,
                "launches_per_step": launches,
                "avg_launch_ms": avg_ms, "algorithmic_flop_per_launch": k_flop[k] / max(launches, 1),
                "share_of_step_time": (k_ms[k] / max(split_steps, 1)) / ms_per_step_with_events if ms_per_step_with_events else None}

    out = {
        "metric": "prefill tokens/s on 1 MI355X (8B-shape, 32k ctx)" if args.workload == "llama8b_32k" and not args.layers and not args.fp8 and not args.few_rows
                  else f"prefill tokens/s on 1 MI355X ({args.workload}" + (", FP8-dynamic linear layers)" if args.fp8 else ")"),
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {I.BF16: "bf16", I.F32: "f32", I.BF16_FP8: "fp8 e4m3 linear layers, bf16 elsewhere"}[cfg.dtype], "data": "synthetic",
        "config": {"workload": args.workload, "layers": cfg.n_layers, "d_model": cfg.d_model,
                   "requests": len(lens), "tokens": tokens, "mlp_chunk": chunk, "packed_rows": args.packed,
                   "few_rows_split": bool(args.few_rows), "weights": "random-init N(0,0.02), seeded"},
        "end_to_end": {"algorithmic_tflop": (lin_f + att_f) / 1e12,
                       "achieved_tflops": (lin_f + att_f) / 1e12 / (ms_per_step / 1e3),
                       "frac_of_bf16_mfma_peak": (lin_f + att_f) / 1e12 / (ms_per_step / 1e3) / PEAK_BF16_TFLOPS},
        "peak_hbm_bytes": {"weights_arena": ctx.weights_bytes, "workspace_arena": ctx.workspace_bytes,
                           "device_in_use_after_run": int(total_b - free_b)},
        "timing": {"value_pass": "no per-launch events", "ms_per_step_with_per_launch_events": ms_per_step_with_events,
                   "per_kernel_split_steps": split_steps},
        "load_seconds": load_s,
        # the nominal MFMA peak assumes 2400 MHz; the board runs this load at its power limit, below that
        "shader_clock_mhz": {"during_untimed_steps": sclk, "nominal": 2400},
        "board_power_w": watts,
    }
    if sum(k_ms.values()) > 0:
        # `roofline` is the kernel with the largest share of the step; the others follow
        order = sorted(classes, key=lambda k: -k_ms[k])
        out["roofline"] = roof(order[0])
        out["roofline_other_kernels"] = [roof(k) for k in order[1:]]
    if args.reuse_prefix > 0:
        # not part of `value`: the same request again with the K/V of its first P tokens cached
        p_len = min(args.reuse_prefix, lens[0] - 1)
        cache_bytes = ctx.po_attach_kv_cache(p_len)
        ctx.po_prefill_prefix(reqs[0], p_len, cand, want_logits=False)          # stores the prefix
        ctx.po_prefill_prefix(reqs[0], 0, cand, want_logits=False)              # warm-up of the reuse path
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            _, _, reused = ctx.po_prefill_prefix(reqs[0], 0, cand, want_logits=False)
        torch.cuda.synchronize()
        out["prefix_reuse"] = {"request_tokens": lens[0], "reused_prefix_tokens": int(reused),
                               "ms_per_request": 1e3 * (time.perf_counter() - t0) / args.steps,
                               "kv_cache_bytes": int(cache_bytes)}
    if args.jct_profile > 0:
        import numpy as np
        n_max = max(lens)
        cache_bytes = ctx.po_attach_kv_cache(n_max - 1)
        t0 = time.perf_counter()
        n_in, n_c, ms = ctx.po_profile_jct(n_max, args.jct_profile)
        wall = time.perf_counter() - t0
        sch = B.Scheduler(0.0)
        c0, c_in, c_cached = sch.po_sched_fit_jct_model(n_in, n_c, ms)
        fit = c0 + c_in * n_in + c_cached * n_c
        ss_res, ss_tot = float(np.sum((ms - fit) ** 2)), float(np.sum((ms - ms.mean()) ** 2))
        out["jct_profile"] = {"max_len": n_max, "step": args.jct_profile, "pairs": int(len(ms)), "profile_seconds": wall,
                              "linear_model_ms": {"c0": c0, "c_input": c_in, "c_cached": c_cached},
                              "linear_model_r2": 1.0 - ss_res / ss_tot,
                              "linear_model_max_abs_err_ms": float(np.max(np.abs(ms - fit))),
                              "pearson_miss_tokens_vs_jct": float(np.corrcoef((n_in - n_c).astype(np.float64), ms)[0, 1]),
                              "jct_ms_min_max": [float(ms.min()), float(ms.max())],
                              "kv_cache_bytes": int(cache_bytes)}
    if args.workload == "llama8b_32k" and not (args.layers or args.fp8 or args.packed or args.few_rows or args.no_extras):
        out["footprint_sweep"] = footprint_sweep(B, I, cfg, chunk, ctx, max(lens))
    ctx.po_destroy()
    del ctx
    torch.cuda.empty_cache()
    if not args.no_extras:
        out["micro_peak"] = micro_peaks(B, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, w["wseed"], w["tseed"], lens, 2, 4096)
        out["cpu_baseline_full"] = [cpu_baseline_full_tiny(), cpu_baseline_recorded()]
        if args.cpu_baseline_request:
            out["cpu_baseline_full"].append(cpu_baseline_full_request())
    print(json.dumps(out))


if __name__ == "__main__":
    main()
