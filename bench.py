#!/usr/bin/env python3
"""Benchmark of the quantized-KV chunk-attention hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input of the Large
configuration (48 heads, head_dim 128, 4096-token chunk, 16 cached chunks at INT2):
    kvq_quantize_append   of the newest cached chunk (the cache is truncated to 15 chunks first,
                          a host-side counter change), then
    kvq_chunk_attention   of the current chunk's 4096 queries over the 65536 cached tokens plus
                          the 4096 unquantized current tokens, with the Taylor correction on.
Inputs are resident in HBM before the timed region.  `value` is the algorithmic attention work
4*H*M*(N_S+N_R)*d per step divided by the whole step time (append included).

Prints ONE JSON line.  Extra fields: per-kernel timings from HIP events recorded on the launch
stream inside the timed region, the correction overhead (corrected vs uncorrected kernel,
interleaved), the roofline of the dominant kernel, and the CPU oracle timed on the host cores on a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16/f16 matrix peak
# Sustained rate of v_mfma_f32_32x32x16_f16 measured on this part with one wave per SIMD
# (profiles/microbench_issue_rates.md): the yardstick for `frac_of_measured_peak`.
MFMA_MEASURED_TFLOPS = 2446.0
HBM_PEAK_GBS = 8000.0
# HBM bytes of one attention launch on the Large workload (per-token INT2, fp32 metadata), from rocprofv3
# FETCH_SIZE / WRITE_SIZE runs of this program scaled by the same counters on a plain 1 GiB elementwise kernel
# (--calibration-copy): 223,500 KiB x 2.000 + 49,920 KiB x 1.000.  A profile figure, not measured by this run:
# it depends on the cache layout and on the placement of workgroups, which have not changed since it was taken
# (profiles/attention_mfma_large_int2_counters.md names the library version).
ATTENTION_TRAFFIC_BYTES_LARGE = 508.8e6
# What the attention kernel computes in: BF16 inputs and outputs; cached scores as FP4 codes x four FP6 query
# pieces on the block-scaled MFMA, current scores and P*V in bf16 MFMA, fp32 accumulation and softmax.
ARITHMETIC = "bf16 I/O; FP4 x FP6 block-scaled MFMA (cached scores), bf16 MFMA (current scores, P*V), fp32 accumulate"
TOL_OUT, TOL_MASS, MASS_FLOOR = 2e-2, 1e-3, 1e-6


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)  # the first launches of a process run 5-20 % slower (clocks ramping up)
    ap.add_argument("--workload", default="large", choices=["small", "mid", "large", "stream"])
    ap.add_argument("--bits", type=int, default=0, choices=[0, 2, 4],
                    help="code width of the cache; 0 = the workload's own (2; the mid workload is also defined at 4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the untimed side measurements (stream, mid INT2 / INT4, large with groups of 32)")
    ap.add_argument("--cpu-heads", type=int, default=8, help="heads (all query rows each) given to the CPU oracle")
    ap.add_argument("--meta", default="fp32", choices=["fp32", "fp8"],
                    help="per-token metadata format of the cache: fp32 scale + zero-point (default, the headline "
                         "configuration) or FP8-E4M3 scale + BF16 zero-point (2.19 bits per element at INT2)")
    ap.add_argument("--group", type=int, default=0, choices=[0, 32, 64],
                    help="channels per (scale, zero-point) group; 0 = one group per token.  Groups of 32 or 64 use "
                         "FP8-E4M3/BF16 metadata (2.75 / 2.375 bits per element at INT2)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="before the warmup, run a plain elementwise kernel over a 1 GiB buffer three times "
                         "(dst = src + 1: reads 1 GiB, writes 1 GiB; outside the timed region): the yardstick "
                         "for FETCH_SIZE / WRITE_SIZE counter runs")
    return ap.parse_args()


def cpu_baseline(w, wl, n_heads, gpu_out=None, gpu_mass=None):
    """The oracle, as it stands, on the first `n_heads` heads of the workload (all query rows, all keys).
    gpu_out [m][H][d], gpu_mass [H][m] (numpy, from the timed configuration): compared with what the oracle
    computes for those heads; returns the baseline record and the parity record."""
    import oracle
    n_heads = min(n_heads, w.num_heads)
    t_att = t_quant = 0.0
    quant_rows = 0
    err_out = err_ps = err_pr = 0.0
    for h in range(n_heads):
        ks, vs = zip(*[wl.chunk_kv(w, c, [h]) for c in range(w.cached_chunks)])
        kc, vc = np.concatenate(ks)[:, 0].astype(np.float64), np.concatenate(vs)[:, 0].astype(np.float64)
        kr, vr = wl.chunk_kv(w, w.cached_chunks, [h])
        q = wl.chunk_q(w, [h])[:, 0]
        t0 = time.perf_counter()
        k_codes, k_scale, k_zero = oracle.quantize(kc, w.bits)
        v_codes, v_scale, v_zero = oracle.quantize(vc, w.bits)
        t_quant += time.perf_counter() - t0
        quant_rows += 2 * kc.shape[0]
        khat, vhat = oracle.dequantize(k_codes, k_scale, k_zero), oracle.dequantize(v_codes, v_scale, v_zero)
        t0 = time.perf_counter()
        o_ref, ps_ref = oracle.attention(q, khat, k_scale, vhat, kr[:, 0], vr[:, 0], correction=1)
        t_att += time.perf_counter() - t0
        if gpu_out is not None:
            err_out = max(err_out, float(np.max(np.abs(gpu_out[:, h, :].astype(np.float64) - o_ref))))
            ps = gpu_mass[h].astype(np.float64)
            for got, ref in ((ps, ps_ref), (1.0 - ps, 1.0 - ps_ref)):
                sel = ref >= MASS_FLOOR
                if np.any(sel):
                    rel = float(np.max(np.abs(got[sel] - ref[sel]) / ref[sel]))
                    if ref is ps_ref:
                        err_ps = max(err_ps, rel)
                    else:
                        err_pr = max(err_pr, rel)
    n_keys = w.cached_tokens + w.chunk_tokens
    flop = 4.0 * n_heads * w.chunk_tokens * n_keys * w.head_dim
    parity = None if gpu_out is None else {
        "heads": n_heads, "rows_per_head": w.chunk_tokens, "max_abs_out": err_out, "max_rel_mass_cached": err_ps,
        "max_rel_mass_current": err_pr, "tol_out": TOL_OUT, "tol_mass_rel": TOL_MASS, "mass_floor": MASS_FLOOR,
        "ok": bool(err_out <= TOL_OUT and max(err_ps, err_pr) <= TOL_MASS)}
    return parity, {
        "value": flop / t_att / 1e12,
        "unit": "TFLOP/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": "attention: %d of %d heads x all %d query rows x all %d keys of the %s config (%.1f s); "
                  "quantizer: the %d cached K/V vectors of those heads (%.1f s)"
                  % (n_heads, w.num_heads, w.chunk_tokens, n_keys, w.name, t_att, quant_rows, t_quant),
        "attention_seconds": t_att,
        "quantize_rows_per_s": quant_rows / t_quant,
        "quantize_gb_per_s_equiv": quant_rows * (w.quantize_bytes(1) / (2 * w.num_heads)) / t_quant / 1e9,
    }


def run_stream(args, torch, B, wl):
    """Stream config: one 4096-token chunk appended 32 times, corrected attention after every append."""
    w = wl.WORKLOADS["stream"]
    dev = "cuda:0"

    def up(x):
        return torch.from_numpy(x).to(dev).to(torch.bfloat16)

    cache = B.Cache(B.make_desc(w.num_heads, w.head_dim, w.bits, w.cached_tokens, B.KVQ_BF16), dev)
    k, v = (up(x) for x in wl.chunk_kv(w, 0))
    q = up(wl.chunk_q(w))
    out = torch.empty_like(q)
    T = w.cached_chunks

    def one_pass(events=None):
        B.kvq_cache_reset(cache)
        for t in range(T):
            if events:
                events[t][0].record()
            B.kvq_quantize_append(cache, k, v)
            if events:
                events[t][1].record()
            B.kvq_chunk_attention(cache, 0, (t + 1) * w.chunk_tokens, q, k, v, out, None, 0.0, 1)
            if events:
                events[t][2].record()

    for _ in range(max(1, args.warmup // 2)):
        one_pass()
    torch.cuda.synchronize()
    steps = max(1, args.steps // 4)
    ev = [[[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(T)] for _ in range(steps)]
    t0 = time.perf_counter()
    for s in range(steps):
        one_pass(ev[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    t_q = np.array([[e[0].elapsed_time(e[1]) for e in p] for p in ev]).mean(axis=0)
    t_a = np.array([[e[1].elapsed_time(e[2]) for e in p] for p in ev]).mean(axis=0)
    flop_t = np.array([4.0 * w.num_heads * w.chunk_tokens * ((t + 2) * w.chunk_tokens) * w.head_dim for t in range(T)])
    total_flop = float(flop_t.sum())
    ms_per_step = wall * 1e3 / steps
    att_tf = total_flop / (t_a.sum() * 1e-3) / 1e12
    return {
        "metric": "corrected INT2-KV chunk-attention TFLOP/s (+ % MFMA peak); quantize GB/s",
        "value": total_flop / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": steps, "warmup": max(1, args.warmup // 2), "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": ARITHMETIC, "data": "synthetic",
        "config": {"workload": "stream: 48 heads, head_dim 128, one 4096-token chunk appended 32 times to the INT2 cache "
                               "(131072 tokens), corrected attention from the chunk's queries after every append",
                   "step": "32 x (quantize_append + chunk_attention)"},
        "quantize_us_per_append": float(t_q.mean() * 1e3),
        "quantize_gb_per_s": w.quantize_bytes() / (t_q.mean() * 1e-3) / 1e9,
        "per_chunk_latency_ms": [float(a + b) for a, b in zip(t_q, t_a)],
        "attention_tflops": att_tf,
        "pct_mfma_peak": 100.0 * att_tf / MFMA_PEAK_TFLOPS,
        "roofline": {"kernel": "attention_mfma_kernel<2, true, %s, false>" % ("true" if args.meta == "fp8" else "false"), "bound": "mfma", "achieved": att_tf,
                     "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": att_tf / MFMA_PEAK_TFLOPS, "traffic": None},
    }


def _events(torch, n):
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def _time_attention(torch, B, cache, n_cached_tokens, q, k_cur, v_cur, out, warm=3, reps=6):
    """Mean time in ms of corrected kvq_chunk_attention calls, from events on the launch stream."""
    for _ in range(warm):
        B.kvq_chunk_attention(cache, 0, n_cached_tokens, q, k_cur, v_cur, out, None, 0.0, 1)
    ev = _events(torch, reps + 1)
    ev[0].record()
    for i in range(reps):
        B.kvq_chunk_attention(cache, 0, n_cached_tokens, q, k_cur, v_cur, out, None, 0.0, 1)
        ev[i + 1].record()
    torch.cuda.synchronize()
    return float(np.mean([ev[i].elapsed_time(ev[i + 1]) for i in range(reps)]))


def _attention_record(w, ms, extra=None):
    tf = w.attention_flop / (ms * 1e-3) / 1e12
    rec = {"attention_ms": ms, "attention_tflops": tf, "frac": tf / MFMA_PEAK_TFLOPS}
    rec.update(extra or {})
    return rec


def side_measurements(torch, B, wl, large_chunks):
    """The other benchmark configurations, each timed with its own events after the headline steps (untimed for
    `value`): the paper's default storage format on the large shape (INT2, groups of 32, FP8/BF16 metadata), the
    mid shape at INT2 and INT4, and one pass of the stream configuration.  large_chunks: the large workload's
    cached and current chunks already on the device, [(k, v)] * 17."""
    dev = "cuda:0"
    res = {}

    def up(x):
        return torch.from_numpy(x).to(dev).to(torch.bfloat16)

    # large, g = 32
    w = wl.WORKLOADS["large"]
    q = up(wl.chunk_q(w))
    out = torch.empty_like(q)
    cache = B.Cache(B.make_desc(w.num_heads, w.head_dim, w.bits, w.cached_tokens, B.KVQ_BF16,
                                meta_format=B.KVQ_META_FP8_BF16, group_size=32), dev)
    ev = _events(torch, 2)
    for c in range(w.cached_chunks):
        if c == w.cached_chunks - 1:
            ev[0].record()
        B.kvq_quantize_append(cache, *large_chunks[c])
    ev[1].record()
    ms = _time_attention(torch, B, cache, w.cached_tokens, q, *large_chunks[w.cached_chunks], out)
    res["large_g32"] = _attention_record(w, ms, {
        "format": "INT2, groups of 32 channels, FP8-E4M3 scale + BF16 zero-point (2.75 bits per element)",
        "quantize_ms": float(ev[0].elapsed_time(ev[1]))})
    del cache

    # mid, INT2 and INT4
    w2 = wl.WORKLOADS["mid"]
    chunks = [tuple(up(x) for x in wl.chunk_kv(w2, c)) for c in range(w2.cached_chunks + 1)]
    q = up(wl.chunk_q(w2))
    out = torch.empty_like(q)
    for bits in (2, 4):
        wb = w2.with_bits(bits)
        cache = B.Cache(B.make_desc(wb.num_heads, wb.head_dim, bits, wb.cached_tokens, B.KVQ_BF16), dev)
        for c in range(wb.cached_chunks):
            B.kvq_quantize_append(cache, *chunks[c])
        ms = _time_attention(torch, B, cache, wb.cached_tokens, q, *chunks[wb.cached_chunks], out)
        res["mid_int%d" % bits] = _attention_record(wb, ms, {"format": "INT%d per token, fp32 metadata" % bits})
        del cache
    del chunks

    # stream: the same chunk appended 32 times, corrected attention after every append; one warm pass, one timed
    w3 = wl.WORKLOADS["stream"]
    k, v = (up(x) for x in wl.chunk_kv(w3, 0))
    q = up(wl.chunk_q(w3))
    out = torch.empty_like(q)
    cache = B.Cache(B.make_desc(w3.num_heads, w3.head_dim, w3.bits, w3.cached_tokens, B.KVQ_BF16), dev)
    T = w3.cached_chunks
    for timed in (False, True):
        B.kvq_cache_reset(cache)
        ev = [_events(torch, 3) for _ in range(T)]
        for t in range(T):
            ev[t][0].record()
            B.kvq_quantize_append(cache, k, v)
            ev[t][1].record()
            B.kvq_chunk_attention(cache, 0, (t + 1) * w3.chunk_tokens, q, k, v, out, None, 0.0, 1)
            ev[t][2].record()
        torch.cuda.synchronize()
    t_q = np.array([e[0].elapsed_time(e[1]) for e in ev])
    t_a = np.array([e[1].elapsed_time(e[2]) for e in ev])
    flop = sum(4.0 * w3.num_heads * w3.chunk_tokens * ((t + 2) * w3.chunk_tokens) * w3.head_dim for t in range(T))
    tf = flop / (t_a.sum() * 1e-3) / 1e12
    res["stream"] = {
        "quantize_us_per_append": float(t_q.mean() * 1e3),
        "quantize_gb_per_s": w3.quantize_bytes() / (t_q.mean() * 1e-3) / 1e9,
        "per_chunk_latency_ms": {"first": float(t_q[0] + t_a[0]), "last": float(t_q[-1] + t_a[-1]),
                                 "sum": float(t_q.sum() + t_a.sum())},
        "attention_tflops": tf, "frac": tf / MFMA_PEAK_TFLOPS,
    }
    return res


def machine_context():
    """Clocks as rocm-smi reports them after the run (None where the tool is not there): lets a reader tell a
    slow machine from a regression."""
    import subprocess
    # Under a profiler every child process is instrumented too (its preloaded library opens the GPU in the child
    # before rocm-smi's own interpreter hop): no children then.
    if any("rocprof" in os.environ.get(k, "").lower() for k in ("LD_PRELOAD", "ROCP_TOOL_LIBRARIES", "ROCPROFILER_REGISTER_FORCE_LOAD")) \
            or any(k.startswith("ROCPROF") for k in os.environ):
        return None
    try:
        r = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True, timeout=20)
        card = next(iter(json.loads(r.stdout).values()))
        return {k: v for k, v in card.items() if "sclk" in k or "mclk" in k}
    except Exception:
        return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (heads shard with no "
              "communication: each GPU would run this same kernel on its share of the heads). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2605_26266_amd import binding as B
    from paper_2605_26266_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    B.lib()  # fail loudly when the library is not built
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.workload == "stream":
        print(json.dumps(run_stream(args, torch, B, wl)))
        return
    w = wl.WORKLOADS[args.workload]
    if args.bits and args.bits != w.bits:
        w = w.with_bits(args.bits)
        args.no_extras = True
    n_cached = w.cached_chunks

    def up(x):
        return torch.from_numpy(x).to(dev).to(torch.bfloat16)

    # ---- resident inputs: the cache filled with chunks 0..n-2, chunk n-1 kept in bf16 for the timed append
    if args.group:
        args.meta = "fp8"
    meta = B.KVQ_META_FP8_BF16 if args.meta == "fp8" else B.KVQ_META_FP32
    n_groups = w.head_dim // args.group if args.group else 1
    cache = B.Cache(B.make_desc(w.num_heads, w.head_dim, w.bits, w.cached_tokens, B.KVQ_BF16, meta_format=meta,
                                group_size=args.group or None), dev)
    extras = not args.no_extras and w.name == "large" and args.meta == "fp32" and not args.group
    chunks = []   # kept on the device for the side measurements (1.6 GB at the large shape)
    for c in range(n_cached - 1):
        k, v = wl.chunk_kv(w, c)
        kv = (up(k), up(v))
        B.kvq_quantize_append(cache, *kv)
        if extras:
            chunks.append(kv)
    k_new, v_new = (up(x) for x in wl.chunk_kv(w, n_cached - 1))
    k_cur, v_cur = (up(x) for x in wl.chunk_kv(w, n_cached))
    chunks += [(k_new, v_new), (k_cur, v_cur)]
    q = up(wl.chunk_q(w))
    out = torch.empty_like(q)
    mass = torch.empty((w.num_heads, w.chunk_tokens), dtype=torch.float32, device=dev)
    keep = (n_cached - 1) * w.chunk_tokens
    torch.cuda.synchronize()

    def step(events=None):
        B.kvq_cache_truncate(cache, keep)
        if events:
            events[0].record()
        B.kvq_quantize_append(cache, k_new, v_new)
        if events:
            events[1].record()
        B.kvq_chunk_attention(cache, 0, w.cached_tokens, q, k_cur, v_cur, out, mass, 0.0, 1)
        if events:
            events[2].record()

    if args.calibration_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(ev[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    t_quant = np.array([e[0].elapsed_time(e[1]) for e in ev])   # ms
    t_att = np.array([e[1].elapsed_time(e[2]) for e in ev])

    # ---- correction overhead: corrected and uncorrected kernels interleaved run by run
    reps = max(5, args.steps // 2)
    pair = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(reps)]
    for p in pair:
        p[0].record()
        B.kvq_chunk_attention(cache, 0, w.cached_tokens, q, k_cur, v_cur, out, mass, 0.0, 1)
        p[1].record()
        B.kvq_chunk_attention(cache, 0, w.cached_tokens, q, k_cur, v_cur, out, mass, 0.0, 0)
        p[2].record()
    torch.cuda.synchronize()
    t_on = np.median([p[0].elapsed_time(p[1]) for p in pair])
    t_off = np.median([p[1].elapsed_time(p[2]) for p in pair])

    flop = w.attention_flop
    q_bytes = w.quantize_bytes(meta_bytes=3 * n_groups if args.meta == "fp8" else 8)
    att_ms = float(np.mean(t_att))
    quant_ms = float(np.mean(t_quant))
    att_tflops = flop / (att_ms * 1e-3) / 1e12
    result = {
        "metric": "corrected INT2-KV chunk-attention TFLOP/s (+ % MFMA peak); quantize GB/s",
        "value": flop / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": ARITHMETIC if not args.group and w.bits == 2 else "bf16 I/O; f16 MFMA (cached scores), bf16 / f16 MFMA (current scores, P*V), fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": "%s: %d heads, head_dim %d, chunk %d tokens, %d cached chunks (%d tokens) INT%d "
                               "%s asymmetric after Hadamard rotation, %s metadata, correction on"
                               % (w.name, w.num_heads, w.head_dim, w.chunk_tokens, n_cached, w.cached_tokens, w.bits,
                                  "group-wise (g = %d)" % args.group if args.group else "per-token",
                                  "FP8-E4M3/BF16" if args.meta == "fp8" else "fp32"),
                   "step": "quantize_append(1 chunk) + chunk_attention"},
        "attention_ms": att_ms,
        "attention_tflops": att_tflops,
        "pct_mfma_peak": 100.0 * att_tflops / MFMA_PEAK_TFLOPS,
        "quantize_ms": quant_ms,
        "quantize_gb_per_s": q_bytes / (quant_ms * 1e-3) / 1e9,
        "quantize_pct_hbm_peak": 100.0 * q_bytes / (quant_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "correction_overhead_pct": 100.0 * (t_on / t_off - 1.0),
        "attention_ms_uncorrected": float(t_off),
        "roofline": {
            "kernel": ("attention_mfma_group_kernel<2, true, %d>" % n_groups if args.group else
                       "attention_mfma_kernel<2, true, %s, false>" % ("true" if args.meta == "fp8" else "false")),
            "bound": "mfma",
            "achieved": att_tflops,
            "peak": MFMA_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": att_tflops / MFMA_PEAK_TFLOPS,
            "frac_of_measured_peak": att_tflops / MFMA_MEASURED_TFLOPS,
            "measured_peak": MFMA_MEASURED_TFLOPS,
            "traffic": ATTENTION_TRAFFIC_BYTES_LARGE if w.name == "large" and args.meta == "fp32" and not args.group and w.bits == 2 else None,
            "traffic_source": "rocprofv3 FETCH_SIZE / WRITE_SIZE profile (profiles/), not measured by this run",
            "attention_ms_min": float(np.min(t_att)), "attention_ms_max": float(np.max(t_att)),
        },
    }
    # The timed configuration once more with the correction on (the overhead pairs end on the uncorrected kernel):
    # its output and cached masses are what the oracle's are compared with below.
    B.kvq_chunk_attention(cache, 0, w.cached_tokens, q, k_cur, v_cur, out, mass, 0.0, 1)
    torch.cuda.synchronize()
    n_par = min(args.cpu_heads, w.num_heads)
    gpu_out = out[:, :n_par].float().cpu().numpy()
    gpu_mass = mass[:n_par].cpu().numpy()
    if extras:
        result.update(side_measurements(torch, B, wl, chunks))
    result["machine"] = machine_context()
    failed = False
    if not args.no_cpu_baseline:
        can_compare = args.meta == "fp32" and not args.group    # the oracle leg quantizes with fp32 metadata
        parity, result["cpu_baseline"] = cpu_baseline(w, wl, args.cpu_heads, gpu_out if can_compare else None, gpu_mass)
        if parity is not None:
            result["parity"] = parity
            result["parity_max_abs_out"] = parity["max_abs_out"]
            result["parity_max_rel_mass"] = max(parity["max_rel_mass_cached"], parity["max_rel_mass_current"])
            failed = not parity["ok"]
    print(json.dumps(result))
    if failed:
        print("bench.py: the timed configuration does not match the oracle within 2e-2 (outputs) / 1e-3 (masses)", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
