#!/usr/bin/env python3
"""Benchmark of the batch-1 decode / prefill path on ONE MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload (benchmark configs[3], the long end of the paper's regime,
Sec. IV-E: LLaMA-2-7B shape, fp16, batch 1): seeded random weights, a
500-token random prompt through the MFMA prefill (TTFT), then K greedy decode
steps as hipGraph replays (KV length 500 -> 500+K).  One "step" is one decode
step = one generated token.  Prints ONE JSON line; progress goes to stderr.

Reported: p50/p99 per-token latency (host wall clock around ll_decode_step),
tokens/s, TTFT for prompts 10..500, device time per step and its HBM roofline
fraction, the dominant kernel's roofline (gate/up GEMV, hipEvent-timed), graph
replay vs eager launches, and the CPU oracle timed on this machine's host cores.
"""
import argparse
import json
import re
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PROMPT_LENGTHS = (10, 25, 50, 100, 250, 500)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def step_bytes(cfg, n_keys):
    """Algorithmic HBM bytes of one decode step attending n_keys keys: every
    fp16 weight once, the gain vectors, one embedding row, K and V rows read,
    one K and one V row written."""
    d, F, V, Lyr = cfg["d_model"], cfg["ffn_hidden"], cfg["vocab"], cfg["n_layers"]
    weights = 2 * (Lyr * (4 * d * d + 3 * d * F) + V * d)
    gains = 2 * (2 * Lyr + 1) * d
    emb = 2 * d
    kv_read = Lyr * 2 * d * 2 * n_keys
    kv_write = Lyr * 2 * d * 2
    return weights + gains + emb + kv_read + kv_write


def gateup_bytes(cfg):
    """Algorithmic bytes of one gate/up GEMV launch: both fp16 matrices, the gain, x in, m out."""
    d, F = cfg["d_model"], cfg["ffn_hidden"]
    return 2 * F * d * 2 + 2 * d + 4 * d + 4 * F


def counter_traffic():
    """HBM bytes per gate/up launch from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE runs of `bench.py --counters`, each scaled by a copy kernel of known size), or None."""
    path = os.path.join(ROOT, "profiles", "counters_decode_gemv_7b.md")
    try:
        with open(path) as f:
            m = re.search(r"^traffic_bytes_per_launch:\s*(\d+)", f.read(), re.M)
        return int(m.group(1)) if m else None
    except OSError:
        return None


def cpu_info():
    """(model name, physical cores, logical CPUs) of the host, from /proc/cpuinfo."""
    model, cores = "unknown", set()
    try:
        phys = core = None
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name") and model == "unknown":
                    model = line.split(":", 1)[1].strip()
                elif line.startswith("physical id"):
                    phys = line.split(":", 1)[1].strip()
                elif line.startswith("core id"):
                    core = line.split(":", 1)[1].strip()
                elif not line.strip():
                    if phys is not None and core is not None:
                        cores.add((phys, core))
                    phys = core = None
    except OSError:
        pass
    return model, (len(cores) or None), os.cpu_count()


def gap_stats(csv_path):
    """Launch gaps from a `rocprofv3 --kernel-trace --output-format csv` kernel trace of a --launch-gaps
    run: for every pair of consecutive kernels (by start time) start(n+1) - end(n) in microseconds;
    negative = the next kernel's first wave started before the previous kernel's last wave ended.  Only
    the decode steps count: the run sleeps 0.3 s between the prefill and the steps, and the trace is cut
    at its last idle gap of more than 0.1 s.  Gaps after a step's last kernel (the token selection) are
    reported apart: they hold the host's round trip between two ll_decode_step calls."""
    import csv
    rows = []
    with open(csv_path, newline="") as f:
        for r in csv.DictReader(f):
            rows.append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]), r["Kernel_Name"]))
    rows.sort()
    cut = 0
    for i in range(len(rows) - 1):
        if rows[i + 1][0] - rows[i][1] > 100_000_000:
            cut = i + 1
    rows = rows[cut:]
    inner, outer = [], []
    for i in range(len(rows) - 1):
        gap = (rows[i + 1][0] - rows[i][1]) / 1e3
        (outer if "sample_kernel" in rows[i][2] else inner).append(gap)
    inner, outer = np.array(inner), np.array(outer)
    durs = np.array([(r[1] - r[0]) / 1e3 for r in rows])
    steps = max(1, len(outer) + 1)
    return dict(kernels=len(rows), decode_steps=steps, kernels_per_step=len(rows) / steps,
                median_kernel_us=float(np.median(durs)), sum_of_kernel_durations_per_step_us=float(durs.sum()) / steps,
                within_step=dict(pairs=int(inner.size), gap_median_us=float(np.median(inner)), gap_p99_us=pct(inner, 99),
                                 gap_max_us=float(inner.max()), gap_min_us=float(inner.min()),
                                 idle_per_step_us=float(inner[inner > 0].sum()) / steps,
                                 overlapping_pairs=int((inner < 0).sum())),
                between_steps=dict(pairs=int(outer.size), gap_median_us=float(np.median(outer)) if outer.size else None,
                                   gap_p99_us=pct(outer, 99) if outer.size else None))


def pct(v, p):
    v = np.sort(np.asarray(v))
    k = max(0, min(len(v) - 1, int(np.ceil(p / 100.0 * len(v))) - 1))   # nearest rank
    return float(v[k])


def batched_leg(cfg, w_t, batch=16):
    """Batched lock-step decoding over the paged KV cache: `batch` sequences with prompts of the sweep's
    lengths, 100 timed steps back to back (device time), then 20 single steps (host wall time)."""
    import numpy as np
    from paper_2604_23467_amd import binding, workloads as wl
    bsess = binding.Session(cfg, w_t)
    blens = [PROMPT_LENGTHS[i % len(PROMPT_LENGTHS)] for i in range(batch)]
    page_tokens, bsteps = 16, 100
    n_pages = sum((n + 5 + bsteps + 20) // page_tokens + 2 for n in blens) + 1    # 5 + bsteps + 20 steps each
    bsess.ll_batch_open(batch, page_tokens, n_pages)
    for i, n in enumerate(blens):
        bsess.ll_batch_add(wl.make_tokens(n, cfg["vocab"], seed=7000 + i))
    for _ in range(5):
        bsess.ll_batch_step()
    kv0 = sum(n + 5 for n in blens)
    b_ms = bsess.ll_batch_dbg_time_steps(bsteps) / bsteps
    hl = np.empty(20)
    for i in range(20):
        t0 = time.perf_counter()
        bsess.ll_batch_step()
        hl[i] = time.perf_counter() - t0
    bsess.ll_batch_close()
    bsess.close()
    # weights once per step whatever the batch; K/V rows of all sequences (mean over the timed steps)
    b_bytes = step_bytes(cfg, 0) + cfg["n_layers"] * 2 * cfg["d_model"] * 2 * (kv0 + batch * (bsteps + 1) // 2 + 2 * batch - 1)
    batched = dict(batch=batch, prompt_lengths=blens, page_tokens=page_tokens, steps=bsteps, ms_per_step=b_ms,
                   tokens_per_s=batch * 1e3 / b_ms, host_p50_us=pct(hl, 50) * 1e6,
                   hbm_tb_per_s=b_bytes / (b_ms * 1e-3) / 1e12)
    log("[bench] batch of %d (prompts 10..500, pages of 16): %.3f ms per step = %.0f tokens/s, %.2f TB/s; "
        "host p50 %.1f us" % (batch, b_ms, batched["tokens_per_s"], batched["hbm_tb_per_s"], batched["host_p50_us"]))
    return batched


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--prompt", type=int, default=500)
    ap.add_argument("--ttft-reps", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-eager", action="store_true")
    ap.add_argument("--cpu-tokens", type=int, default=8)
    ap.add_argument("--counters", action="store_true",
                    help="short run for `rocprofv3 --pmc`: a 256 MiB device copy as the counter "
                         "calibration, then prefill + the decode steps; no timing, no JSON")
    ap.add_argument("--persistent-trace", action="store_true",
                    help="one decode step of the single-persistent-kernel mode with its in-kernel phase "
                         "timestamps (workgroup 0): where a phase's time goes between entry, staging, "
                         "dot products, stores and the grid barrier")
    ap.add_argument("--lib-gemm", action="store_true",
                    help="context only: time torch.matmul (the vendor GEMM library) on the four projection "
                         "shapes at M = 64..512 rows, weights rotated over 8 copies so they stream from HBM")
    ap.add_argument("--batched", action="store_true",
                    help="only the batched-decoding legs (16 and 32 sequences over the paged KV cache): one JSON line")
    ap.add_argument("--launch-gaps", choices=("7b-graph", "7b-eager", "tiny-graph", "tiny-eager"), default=None,
                    help="workload for `rocprofv3 --kernel-trace`: a prefill, then --steps decode steps issued as "
                         "graph replays or as eager launches, on the 7B shape or on the tiny model; nothing else runs")
    ap.add_argument("--decode-variants", action="store_true",
                    help="workload for `rocprofv3 --kernel-trace --stats`: prefill(--prompt) + --steps decode steps in each "
                         "of the measured arrangements of a step (two kernels for attention and O projection, the "
                         "fused launch, the single persistent kernel); prints device ms per step of each")
    ap.add_argument("--gap-stats", metavar="KERNEL_TRACE_CSV", default=None,
                    help="no GPU work: launch-gap statistics of the decode steps in a kernel-trace CSV of a "
                         "--launch-gaps run (JSON on stdout)")
    ap.add_argument("--sweep", type=int, default=0, metavar="REPS",
                    help="latency sweep instead of the default run: for every prompt length in "
                         "{10,25,50,100,250,500}, REPS repetitions (token seed 1000*len + rep) of reset + "
                         "prefill + --steps decode steps; prints TTFT and per-token p50/p99 per length")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (batch-1 latency path, no sharding or "
              "collectives); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    if args.gap_stats:
        print(json.dumps(gap_stats(args.gap_stats)))
        return 0

    import torch
    from paper_2604_23467_amd import binding, workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if args.lib_gemm:
        out = {"metric": "vendor-library GEMM on the prefill projection shapes (context for the hand-written GEMM)",
               "unit": "us", "dtype": "f16", "rows": {}}
        shapes = {"qkv": (12288, 4096), "o": (4096, 4096), "gateup": (22016, 4096), "down": (4096, 11008)}
        for m in (64, 128, 256, 512):
            row = {}
            for name, (n_, k_) in shapes.items():
                ws = [torch.randn(n_, k_, device="cuda:0", dtype=torch.float16) for _ in range(8)]
                x = torch.randn(m, k_, device="cuda:0", dtype=torch.float16)
                for w_ in ws:
                    torch.matmul(x, w_.t())
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(4):
                    for w_ in ws:
                        torch.matmul(x, w_.t())
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / 32
                row[name] = {"us": us, "tflops": 2.0 * m * n_ * k_ / us / 1e6}
                del ws
            out["rows"][str(m)] = row
            log("[bench] library GEMM, M = %3d: %s" % (m, "; ".join("%s %.1f us (%.0f TFLOP/s)" % (k, v["us"], v["tflops"]) for k, v in row.items())))
        print(json.dumps(out), flush=True)
        return 0
    if args.launch_gaps:
        shape, how = args.launch_gaps.split("-")
        flags = binding.LL_FLAG_EAGER if how == "eager" else 0
        if shape == "tiny":
            gcfg = wl.tiny_cfg(max_seq=1024)
            gw = wl.weights_to_torch(wl.make_weights_numpy(gcfg, seed=0), device="cuda:0", dtype=torch.float16)
        else:
            gcfg = wl.llama7b_cfg(max_seq=1024)
            gw = wl.make_weights_torch(gcfg, seed=0, device="cuda:0")
        gs = binding.Session(gcfg, gw, flags=flags)
        gs.ll_prefill(wl.make_tokens(10, gcfg["vocab"], seed=0))
        gs.ll_decode_n(5)
        torch.cuda.synchronize()
        time.sleep(0.3)                      # the idle gap the trace is cut at
        lat = np.empty(args.steps)
        for i in range(args.steps):
            t0 = time.perf_counter()
            gs.ll_decode_step()
            lat[i] = time.perf_counter() - t0
        gs.close()
        print(json.dumps(dict(workload=args.launch_gaps, steps=args.steps, host_p50_us=pct(lat, 50) * 1e6,
                              host_p99_us=pct(lat, 99) * 1e6)), flush=True)
        return 0

    K, W, n_prompt = args.steps, args.warmup, args.prompt
    cfg = wl.llama7b_cfg(max_seq=max(1024, n_prompt + max(K, W) + 64))
    log("[bench] drawing 7B-shaped fp16 weights on the GPU ...")
    w_t = wl.make_weights_torch(cfg, seed=0, device="cuda:0")
    torch.cuda.synchronize()
    prompt = wl.make_tokens(n_prompt, cfg["vocab"], seed=0)

    if args.decode_variants:
        out = {}
        for name, fl in (("default: attention and O projection as two kernels", 0),
                         ("LL_FLAG_FUSED_ATTN_OPROJ: one launch for both", binding.LL_FLAG_FUSED_ATTN_OPROJ),
                         ("LL_FLAG_PERSISTENT: the whole step as one kernel", binding.LL_FLAG_PERSISTENT)):
            vs = binding.Session(cfg, w_t, flags=fl)
            vs.ll_prefill(prompt)
            vs.ll_decode_n(10)
            out[name] = vs.ll_dbg_time_decode(K) / K
            vs.close()
            log("[bench] %-55s %.4f ms per step (device, KV %d..%d)" % (name, out[name], n_prompt + 10, n_prompt + 10 + K))
        print(json.dumps(dict(metric="decode step, measured arrangements", unit="ms", steps=K, prompt=n_prompt, device_ms_per_step=out)))
        return 0

    if args.batched:
        print(json.dumps(dict(metric="batched decode step over a paged KV cache", unit="ms", n_gpus=1, dtype="f16",
                              data="synthetic", legs=[batched_leg(cfg, w_t, 16), batched_leg(cfg, w_t, 32)])))
        return 0

    if args.counters:
        sess = binding.Session(cfg, w_t, flags=binding.LL_FLAG_EAGER)
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        b = torch.empty_like(a)
        b.copy_(a)                                   # known traffic: 256 MiB read + 256 MiB written
        torch.cuda.synchronize()
        binding.ll_dbg_stream_copy(b, a)             # same, through the GEMVs' 16-byte streaming loads
        sess.ll_prefill(prompt)
        sess.ll_decode_n(K)
        sess.close()
        log("[bench] counter run done (%d decode steps after a %d-token prompt)" % (K, n_prompt))
        return 0

    if args.persistent_trace:
        ps = binding.Session(cfg, w_t, flags=binding.LL_FLAG_PERSISTENT)
        ps.ll_prefill(prompt)
        ps.ll_decode_n(5)
        dev_ms = ps.ll_dbg_time_decode(100) / 100
        ps.ll_dbg_trace_decode()
        t = ps.ll_dbg_trace_decode()                 # [phases][8] microseconds since the step's first stamp
        ps.close()
        names = ["qkv", "attn", "oproj", "gateup", "down"]
        nl = cfg["n_layers"]
        rows = {}
        for k, nm in enumerate(names):
            ph = np.array([t[5 * l + k] for l in range(2, nl - 1)])
            nxt = np.array([t[5 * l + k + 1, 0] for l in range(2, nl - 1)])
            staged = ph[:, 1] if (ph[:, 1] >= 0).all() else ph[:, 0]      # attention stages nothing: slot unused
            rows[nm] = {"phase_us": float((nxt - ph[:, 0]).mean()),
                        "entry_to_staged_us": float((staged - ph[:, 0]).mean()),
                        "staged_to_dots_done_us": float((ph[:, 2] - staged).mean()),
                        "dots_done_to_stored_us": float((ph[:, 3] - ph[:, 2]).mean()),
                        "stored_to_barrier_passed_us": float((ph[:, 4] - ph[:, 3]).mean())}
            log("[bench] persistent kernel, phase %-7s %.2f us: staging %.2f, dot products %.2f, stores %.2f, "
                "barrier %.2f" % (nm, rows[nm]["phase_us"], rows[nm]["entry_to_staged_us"],
                                  rows[nm]["staged_to_dots_done_us"], rows[nm]["dots_done_to_stored_us"],
                                  rows[nm]["stored_to_barrier_passed_us"]))
        out = {"metric": "phase timeline of the single persistent decode kernel (workgroup 0, mean over layers 2..30)",
               "unit": "us", "device_ms_per_step": dev_ms, "step_us_by_trace": float(t[-1, 4] - t[0, 0]),
               "phases": rows, "config": {"workload": "7B shape, prompt %d, KV %d" % (n_prompt, n_prompt + 106)}}
        log("[bench] persistent kernel: %.3f ms/step on the device" % dev_ms)
        print(json.dumps(out), flush=True)
        return 0

    sess = binding.Session(cfg, w_t)
    decode_mode = ("persistent-kernel graph", "multi-kernel graph", "eager")[sess.ll_decode_mode()]
    log("[bench] init done; warm-up: prefill(%d) + %d steps" % (n_prompt, W))
    sess.ll_prefill(prompt)
    if W > 0:
        sess.ll_decode_n(W)
    sess.ll_reset()

    if args.sweep > 0:
        out = {"metric": "latency sweep: TTFT and per-token latency p50/p99 per prompt length", "unit": "us",
               "n_gpus": 1, "reps": args.sweep, "decode_steps": K, "decode_mode": decode_mode,
               "dtype": "f16", "data": "synthetic", "lengths": {}}
        for n in PROMPT_LENGTHS:
            tt, lat = np.empty(args.sweep), np.empty((args.sweep, K))
            for r in range(args.sweep):
                p = wl.make_tokens(n, cfg["vocab"], seed=wl.sweep_token_seed(n, r))
                sess.ll_reset()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                sess.ll_prefill(p)
                tt[r] = time.perf_counter() - t0
                for i in range(K):
                    t0 = time.perf_counter()
                    sess.ll_decode_step()
                    lat[r, i] = time.perf_counter() - t0
            dec = [pct(lat[:, K * j // 10:K * (j + 1) // 10].ravel(), 99) * 1e6 for j in range(10)]
            out["lengths"][str(n)] = {
                "ttft_p50_ms": pct(tt, 50) * 1e3, "ttft_p99_ms": pct(tt, 99) * 1e3,
                "token_p50_us": pct(lat.ravel(), 50) * 1e6, "token_p99_us": pct(lat.ravel(), 99) * 1e6,
                "token_max_us": float(lat.max()) * 1e6, "samples": int(lat.size),
                "token_p99_us_by_generation_decile": dec}
            log("[bench] sweep prompt %4d: TTFT p50 %.3f ms p99 %.3f ms | token p50 %.1f us p99 %.1f us (%d samples)"
                % (n, pct(tt, 50) * 1e3, pct(tt, 99) * 1e3, pct(lat.ravel(), 50) * 1e6,
                   pct(lat.ravel(), 99) * 1e6, lat.size))
        sess.close()
        print(json.dumps(out), flush=True)
        return 0

    # ---- TTFT per prompt length (host wall clock of ll_prefill, ids in host memory)
    ttft = {}
    for n in PROMPT_LENGTHS:
        if n > sess.ll_max_prompt():
            continue
        ts = []
        for r in range(args.ttft_reps + 1):
            p = wl.make_tokens(n, cfg["vocab"], seed=wl.sweep_token_seed(n, r))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            sess.ll_prefill(p)
            ts.append((time.perf_counter() - t0) * 1e3)
            sess.ll_reset()
        ttft[n] = float(np.median(ts[1:]))
        log("[bench] TTFT prompt %4d: %.3f ms" % (n, ttft[n]))

    # ---- timed region: K decode steps after the prompt
    sess.ll_prefill(prompt)
    torch.cuda.synchronize()
    lat = np.empty(K)
    t_begin = time.perf_counter()
    for i in range(K):
        t0 = time.perf_counter()
        sess.ll_decode_step()
        lat[i] = time.perf_counter() - t0
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t_begin
    ms_per_step = t_total * 1e3 / K
    p50, p99 = pct(lat, 50) * 1e6, pct(lat, 99) * 1e6
    log("[bench] %d steps: %.3f ms/step host wall, p50 %.1f us, p99 %.1f us" % (K, ms_per_step, p50, p99))

    # ---- device time per step (one event pair around K replays, no host sync in between)
    sess.ll_reset()
    sess.ll_prefill(prompt)
    dev_ms = sess.ll_dbg_time_decode(K) / K
    mean_keys = n_prompt + 1 + (K - 1) / 2.0
    bytes_step = step_bytes(cfg, mean_keys)
    step_gbs = bytes_step / (dev_ms * 1e-3) / 1e9
    log("[bench] device %.3f ms/step -> %.0f GB/s = %.1f%% of %.0f GB/s"
        % (dev_ms, step_gbs, 100 * step_gbs / HBM_PEAK_GBS, HBM_PEAK_GBS))
    # the chip's own streaming ceiling in this run: a read-only pass over 2 GiB with the GEMVs' loads
    big = torch.empty(2 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
    stream_gbs = max(binding.ll_dbg_stream_read(big, reps=4) for _ in range(3))
    del big
    log("[bench] read-only streaming pass over 2 GiB: %.0f GB/s (%.1f%% of nominal); the step runs at %.1f%% of it"
        % (stream_gbs, 100 * stream_gbs / HBM_PEAK_GBS, 100 * step_gbs / stream_gbs))

    # ---- per-kernel-class durations: each class launched back to back over all layers
    #      (every layer's own weights, nothing re-read from cache) between one hipEvent
    #      pair on the library's stream
    sess.ll_reset()
    sess.ll_prefill(prompt)
    sess.ll_decode_n(max(1, min(K, 250)))            # KV length in the middle of the timed range
    prof = {}
    for name, per_step in (("qkv", cfg["n_layers"]), ("attn", cfg["n_layers"]), ("oproj", cfg["n_layers"]),
                           ("gateup", cfg["n_layers"]), ("down", cfg["n_layers"]), ("lmhead", 1)):
        try:
            prof[name] = (sess.ll_dbg_time_kernel_class(name, 4 if per_step > 1 else 32), per_step)
        except binding.LLError:              # a class without launches of its own in this instance
            continue
        log("[bench]   %-7s %8.2f us x %d" % (name, prof[name][0], per_step))
    sess.ll_reset()
    gu_us = prof["gateup"][0]
    gu_gbs = gateup_bytes(cfg) / (gu_us * 1e-6) / 1e9
    kernel_sum_ms = sum(us * n for us, n in prof.values()) / 1e3
    sess.close()

    # ---- graph replay vs eager launches (same kernels, per-kernel dispatch from the host)
    eager = None
    if not args.no_eager:
        es = binding.Session(cfg, w_t, flags=binding.LL_FLAG_EAGER)
        es.ll_prefill(prompt[:10])
        es.ll_decode_n(10)
        el = np.empty(100)
        for i in range(100):
            t0 = time.perf_counter()
            es.ll_decode_step()
            el[i] = time.perf_counter() - t0
        es.close()
        gs = binding.Session(cfg, w_t)
        gs.ll_prefill(prompt[:10])
        gs.ll_decode_n(10)
        gl = np.empty(100)
        for i in range(100):
            t0 = time.perf_counter()
            gs.ll_decode_step()
            gl[i] = time.perf_counter() - t0
        # in-graph stochastic sampling (temperature 0.8, top-k 50, top-p 0.95) against greedy, same session
        gs.ll_reset()
        gs.ll_set_sampling(0.8, 50, 0.95, 1234)
        gs.ll_prefill(prompt[:10])
        gs.ll_decode_n(10)
        sl = np.empty(100)
        for i in range(100):
            t0 = time.perf_counter()
            gs.ll_decode_step()
            sl[i] = time.perf_counter() - t0
        sampling = dict(temperature=0.8, top_k=50, top_p=0.95, p50_us=pct(sl, 50) * 1e6, p99_us=pct(sl, 99) * 1e6,
                        greedy_p50_us=pct(gl, 50) * 1e6)
        log("[bench] prompt 10, 100 steps with top-k/top-p sampling in the graph: p50 %.1f us p99 %.1f us (greedy p50 %.1f us)"
            % (sampling["p50_us"], sampling["p99_us"], sampling["greedy_p50_us"]))
        gs.close()
        # the paper's mechanism: one graph per KV length, rolling buffer, next length captured during the replay
        ls = binding.Session(cfg, w_t, flags=binding.LL_FLAG_PER_LENGTH_GRAPHS)
        ls.ll_prefill(prompt[:10])
        ls.ll_decode_n(10)
        ll = np.empty(100)
        for i in range(100):
            t0 = time.perf_counter()
            ls.ll_decode_step()
            ll[i] = time.perf_counter() - t0
        gstats = ls.ll_dbg_graph_stats()
        ls.close()
        n_cap = gstats["blocking_captures"] + gstats["overlapped_captures"]
        per_length = dict(p50_us=pct(ll, 50) * 1e6, p99_us=pct(ll, 99) * 1e6, graphs_captured=n_cap,
                          capture_ms_per_graph=gstats["capture_ms"] / max(n_cap, 1),
                          blocking_captures=gstats["blocking_captures"])
        log("[bench] prompt 10, 100 steps, one graph per KV length (buffer of 8, capture overlapped with replay): "
            "p50 %.1f us p99 %.1f us, %.2f ms of host time per captured graph"
            % (per_length["p50_us"], per_length["p99_us"], per_length["capture_ms_per_graph"]))
        batched = [batched_leg(cfg, w_t, 16), batched_leg(cfg, w_t, 32)]
        ps = binding.Session(cfg, w_t, flags=binding.LL_FLAG_PERSISTENT)
        ps.ll_prefill(prompt[:10])
        ps.ll_decode_n(10)
        pl = np.empty(100)
        for i in range(100):
            t0 = time.perf_counter()
            ps.ll_decode_step()
            pl[i] = time.perf_counter() - t0
        ps.close()
        eager = dict(prompt=10, steps=100, eager_p50_us=pct(el, 50) * 1e6, eager_p99_us=pct(el, 99) * 1e6,
                     graph_p50_us=pct(gl, 50) * 1e6, graph_p99_us=pct(gl, 99) * 1e6,
                     persistent_kernel_p50_us=pct(pl, 50) * 1e6, persistent_kernel_p99_us=pct(pl, 99) * 1e6,
                     sampling=sampling, per_length_graphs=per_length, batched_decode=batched)
        log("[bench] prompt 10, 100 steps: graph p50 %.1f us p99 %.1f us | eager p50 %.1f us p99 %.1f us | "
            "one persistent kernel p50 %.1f us p99 %.1f us"
            % (eager["graph_p50_us"], eager["graph_p99_us"], eager["eager_p50_us"], eager["eager_p99_us"],
               eager["persistent_kernel_p50_us"], eager["persistent_kernel_p99_us"]))

    # ---- CPU oracle on this machine's host cores (bounded sample; a reported baseline, not the target)
    cpu = None
    if not args.no_cpu_baseline:
        from oracle.cpu_oracle import Oracle
        log("[bench] copying weights to the host for the CPU oracle ...")
        w_np = wl.weights_to_numpy(w_t)
        om = Oracle("f32").model(cfg, w_np)
        om.step(int(prompt[0]))                      # first touch, untimed
        n_tok = args.cpu_tokens
        t0 = time.perf_counter()
        for t in prompt[1:1 + n_tok]:
            om.step(int(t))
        cpu_s = (time.perf_counter() - t0) / n_tok
        om.close()
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        model, phys, logical = cpu_info()
        cpu = dict(value=cpu_s * 1e6, unit="us/token", cores=threads, kind="oracle", cpu_model=model,
                   physical_cores=phys, logical_cpus=logical,
                   sample="%d token passes of the 7B-shaped fp32 oracle (positions 1..%d of the prompt, "
                          "per-token cost is almost independent of KV length)" % (n_tok, n_tok))
        log("[bench] CPU oracle: %.3f s/token on %d threads" % (cpu_s, threads))

    out = {
        "metric": "per-token decode latency p50/p99 (us) + % peak HBM BW; TTFT at 10-500 prompt",
        "value": p50,
        "unit": "us",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "LLaMA-2-7B shape (32 layers, d 4096, 32x128 heads, FFN 11008, vocab 32000), "
                               "fp16 N(0,0.02) weights seed 0, batch 1, %d-token random prompt, %d greedy "
                               "decode steps as hipGraph replays (KV %d -> %d)"
                               % (n_prompt, K, n_prompt, n_prompt + K),
                   "prompt_len": n_prompt, "decode_steps": K},
        "decode_mode": decode_mode,
        "p50_us": p50,
        "p99_us": p99,
        "tokens_per_s": 1e3 / ms_per_step,
        "ttft_ms": {str(k): v for k, v in ttft.items()},
        "step": {"device_ms": dev_ms, "bytes": bytes_step, "achieved_GBps": step_gbs,
                 "frac_of_peak_hbm": step_gbs / HBM_PEAK_GBS, "target_frac_of_peak_hbm": 0.70,
                 "meets_target": bool(step_gbs / HBM_PEAK_GBS >= 0.70),
                 "measured_stream_GBps": stream_gbs, "frac_of_measured_stream": step_gbs / stream_gbs,
                 "sum_of_kernels_ms": kernel_sum_ms},
        "roofline": {"kernel": "gemv_kernel<GATEUP> (RMSNorm + gate/up GEMV + SwiGLU)", "bound": "hbm",
                     "achieved": gu_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gu_gbs / HBM_PEAK_GBS, "traffic": counter_traffic(),
                     "traffic_source": "profiles/counters_decode_gemv_7b.md: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs "
                                       "of `bench.py --counters`, scaled by a copy of known size; a committed "
                                       "figure, not measured by this run",
                     "bytes_per_launch": gateup_bytes(cfg), "avg_us": gu_us},
        "kernels_us": {k: {"avg_us": us, "launches_per_step": n} for k, (us, n) in prof.items()},
        "graph_vs_eager": eager,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
