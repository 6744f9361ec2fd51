#!/usr/bin/env python3
"""Benchmark of the SKVQ hot path on one MI355X.

A step is one generated token of a 7B-shaped model: for each of `--layers` attention layers
(each with its own cache, so that no layer's data is still in the 256 MB Infinity Cache when
its turn comes again) the token leaving the fp16 window is quantized and the new query attends
over the whole cache: one skvq_append_decode_attention call per layer (with --two-calls:
skvq_quantize_append, then skvq_decode_attention; the other way is timed too and reported
beside).  Inputs are seeded synthetic tensors already resident in HBM.

Prints ONE JSON line.  `value` is microseconds per token (all layers) of the headline workload;
`roofline` prices the algorithmic bytes of one layer's attention call against the 8 TB/s HBM
peak, its duration measured with HIP events around the layers' calls issued back to back;
`configs` holds the same measurements for the other baseline configurations (one layer-call
each; the batch-16 one as the prefill followed by 64 append + attention steps); `cpu_baseline`
is the CPU oracle timed on a bounded sample of the same workload.

`--probe NAME` runs a workload for a profiler instead (`rocprofv3 ... -- python3 bench.py --probe
decode`) and prints plain text: `decode` (a few decode calls and a 256 MiB copy, the yardstick of
the traffic counters), `prefill` (prefill-quantize calls back to back), `prefill-attention`, `read` (the library's read-only kernel over slices
of the decode call's size).
"""
from __future__ import annotations

import argparse
import dataclasses
import glob
import hashlib
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_F16_PEAK_FLOPS = 2.5e15
D = 128
HEADLINE = "c3_mistral7b_128k"
OTHER_CONFIGS = ("c1_mha4_2k", "c2_llama7b_32k", "c4_llama7b_1m", "c5_batch16_32k")
C5_DECODE_STEPS = 64  # the batch-16 configuration: decode steps after the prefill

META_BYTES = {"f32": 4, "f16": 2, "e4m3": 1}
MULTI_TOKENS = (2, 4)  # query tokens per call timed for skvq_decode_attention_multi


# ------------------------------------------------------------------ byte model ----

def code_bytes_per_row(w) -> int:
    """Packed key row + the token's share of its V block, bytes per (token, kv head)."""
    return {2.0: 32, 3.0: 48, 4.0: 64}[w.k_bits] + {1.5: 26, 2.0: 32, 3.0: 48, 4.0: 64}[w.v_bits]


def algorithmic_bytes_decode(w, n_tokens: int, n_sink: int = 0, meta: str = "f32") -> int:
    """Bytes one decode call must move: packed rows (K 32|64 B + V 26|32|64 B + two fp32
    (or fp16 / FP8) (scale, zero) pairs per group each), the fp16 ring and sink rows, the query
    and the fp32 output."""
    nq = max(n_tokens - w.window - n_sink, 0)
    nwin = n_tokens - nq
    ng = D // w.group_size
    per_row = code_bytes_per_row(w) + 2 * (2 * META_BYTES[meta] * ng)
    return (w.batch * w.n_kv_heads * (nq * per_row + nwin * 2 * D * 2)
            + w.batch * w.n_q_heads * D * (2 + 4))


def algorithmic_bytes_prefill(w, meta: str = "f32") -> int:
    """Bytes one prefill-quantize call must move: the fp16 K and V read once, the packed rows and the
    fp16 window written."""
    nq = max(w.context - w.window, 0)
    per_row = code_bytes_per_row(w) + 4 * META_BYTES[meta] * (D // w.group_size)
    return w.batch * w.n_kv_heads * (w.context * 2 * D * 2 + nq * per_row + min(w.context, w.window) * 2 * D * 2)


def read_write_yardstick(B, torch, w, device, budget_bytes: int = 9 << 30) -> dict:
    """The library's read/write kernel on the prefill quantizer's traffic: as many bytes read as the call's
    fp16 K and V, a seventh of that written (the packed codes are 1/6.9 of it), rotating through distinct
    buffers so that every launch finds cold data."""
    ratio = 7
    read_bytes = w.batch * w.n_kv_heads * w.context * 2 * D * 2
    write_bytes = (read_bytes // ratio) & ~0xFFF
    n_bufs = int(max(1, min(8, budget_bytes // (ratio * write_bytes))))
    src = torch.ones(n_bufs * ratio * write_bytes, dtype=torch.uint8, device=device)
    dst = torch.empty(n_bufs * write_bytes, dtype=torch.uint8, device=device)
    pairs = [(src[j * ratio * write_bytes:(j + 1) * ratio * write_bytes], dst[j * write_bytes:(j + 1) * write_bytes])
             for j in range(n_bufs)]

    def sweep():
        for s_, d_ in pairs:
            B.skvq_read_write_yardstick(s_, d_, ratio)
    us = float(timed_us(sweep, n_bufs, 5).mean())
    moved = (ratio + 1) * write_bytes
    del src, dst, pairs
    return {"read_bytes": ratio * write_bytes, "write_bytes": write_bytes, "us_per_launch": us,
            "gbps": moved / us / 1e3, "frac_of_hbm_peak": moved / us / 1e3 / HBM_PEAK_GBPS,
            "what": "skvq_read_write_yardstick: the prefill call's fp16 bytes read, a seventh of that written, "
                    "nothing computed, launches back to back on cold data"}


# ------------------------------------------------------- facts from profiles/ ----

def source_fingerprint() -> str:
    """Hash of the kernel sources: profile summaries carry the one they were taken with."""
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2405_06219_amd", "csrc", "*.h*"))):
        with open(path, "rb") as f:
            h.update(os.path.basename(path).encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def profile_facts(workload: str) -> dict:
    """`# key: value` lines of the committed profile summaries of one workload's decode call."""
    facts = {}
    for kind in ("pmc", "kernel_trace"):
        path = os.path.join(ROOT, "profiles", f"decode_{workload}_{kind}.txt")
        if not os.path.exists(path):
            continue
        one = {}
        with open(path) as f:
            for line in f:
                if line.startswith("# ") and ": " in line:
                    key, val = line[2:].rstrip("\n").split(": ", 1)
                    one[key.strip()] = val.strip()
        facts[kind] = one
    return facts


# ------------------------------------------------------------------ GPU side ----

def build_layers(w, n_layers: int, headroom: int, device, n_sink: int = 0, meta: str = "f32", group_bounds=None,
                 keep_sources: bool = False):
    """Per layer: a cache prefilled with w.context seeded synthetic tokens.  Returns the caches,
    the K/V channel scales on the device, each prefill call's duration (HIP events, us) and, if asked
    for, the layers' fp16 sources."""
    import torch
    from paper_2405_06219_amd import binding as B
    from paper_2405_06219_amd import synth

    sk, sv = synth.channel_scales(w)
    sk_d = torch.from_numpy(sk).to(device)[None, :, None, :]
    sv_d = torch.from_numpy(sv).to(device)[None, :, None, :]
    ck, cv = synth.make_clip(w)
    caches, prefill_us, sources = [], [], []
    for layer in range(n_layers):
        # seeded synthetic K/V and the reorder index from their channel ranges (offline calibration stand-in)
        k, v, pk, pv = synth.make_kv_device(w, device, stream=layer)
        # (packed capacity in whole 64-token tiles: every kv head's rows then start on a cache line)
        c = B.SkvqCache(w.batch, w.n_q_heads, w.n_kv_heads, w.group_size, w.v_bits, w.window,
                        -(-(w.context - w.window + headroom) // 64) * 64, pk, pv, ck, cv, device=device, n_sink=n_sink,
                        meta=meta, k_bits=w.k_bits, group_bounds=group_bounds, max_new_tokens=MULTI_TOKENS[-1])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        c.skvq_prefill_quantize(k, v)
        e1.record()
        torch.cuda.synchronize()
        prefill_us.append(e0.elapsed_time(e1) * 1e3)
        if keep_sources:
            sources.append((k, v))
        del k, v
        caches.append(c)
    return caches, (sk_d, sv_d), prefill_us, sources


def timed_us(fn, n_calls: int, reps: int, warm: int = 1) -> np.ndarray:
    """`fn()` issues n_calls library calls back to back; one pair of HIP events around them (a pair
    around every single call would add about 2 us to each).  Returns us per call, one entry per repetition."""
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    out = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        out.append(e0.elapsed_time(e1) * 1e3 / n_calls)
    return np.array(out)


def measure_config(name: str, device, steps: int) -> dict:
    """One of the other baseline configurations: prefill-quantize and one decode step per layer-call
    (enough layers that the calls' data exceeds the Infinity Cache), HIP events around the calls issued
    back to back.  The batch-16 configuration: its prefill, then 64 append + attention steps."""
    import torch
    from paper_2405_06219_amd import binding as B
    from paper_2405_06219_amd import synth

    w = synth.WORKLOADS[name]
    per_call = algorithmic_bytes_decode(w, w.context)
    n_layers = int(min(32, max(1, -(-640_000_000 // per_call))))
    n_steps = C5_DECODE_STEPS if name == "c5_batch16_32k" else max(steps, 4)
    headroom = 2 * n_steps + 16
    caches, (sk_d, sv_d), first_prefill_us, sources = build_layers(w, n_layers, headroom, device, keep_sources=True)
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed)
    q = torch.randn((n_layers, w.batch, w.n_q_heads, D), generator=gen, device=device).to(torch.float16)
    kn = (torch.randn((n_layers, w.batch, w.n_kv_heads, D), generator=gen, device=device) * sk_d[:, :, 0]).to(torch.float16)
    vn = (torch.randn((n_layers, w.batch, w.n_kv_heads, D), generator=gen, device=device) * sv_d[:, :, 0]).to(torch.float16)
    out = torch.empty((n_layers, w.batch, w.n_q_heads, D), dtype=torch.float32, device=device)

    # prefill again, the layers' calls back to back (a cache may be prefilled any number of times)
    def prefill_all():
        for c, (k, v) in zip(caches, sources):
            c.skvq_prefill_quantize(k, v)
    pre = timed_us(prefill_all, n_layers, 3, warm=0)
    del sources
    torch.cuda.empty_cache()

    def step():
        for i, c in enumerate(caches):
            c.skvq_append_decode_attention(kn[i], vn[i], q[i], out_f32=out[i])

    def decode_only():
        for i, c in enumerate(caches):
            c.skvq_decode_attention(q[i], out_f32=out[i])
    if name == "c5_batch16_32k":
        # the 64 decode steps the configuration names, timed as one run
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n_steps):
            step()
        e1.record()
        torch.cuda.synchronize()
        one = np.array([e0.elapsed_time(e1) * 1e3 / (n_steps * n_layers)])
    else:
        one = timed_us(step, n_layers, n_steps)
    dec = timed_us(decode_only, n_layers, max(n_steps // 4, 3))
    n_tokens = w.context + n_steps // 2
    alg = algorithmic_bytes_decode(w, n_tokens)
    pre_alg = algorithmic_bytes_prefill(w)
    res = {
        "shape": {"batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads, "context": w.context,
                  "k_bits": w.k_bits, "v_bits": w.v_bits, "group_size": w.group_size, "window": w.window},
        "layers_rotated": n_layers,
        "decode_step_us": float(one.mean()), "decode_step_us_min": float(one.min()),
        "decode_step": "skvq_append_decode_attention, one call per layer",
        "decode_steps_timed": int(n_steps),
        "decode_only_call_us": float(dec.mean()),
        "decode_algorithmic_bytes": alg,
        "decode_hbm_gbps": alg / (one.mean() * 1e-6) / 1e9,
        "decode_frac_of_hbm_peak": alg / (one.mean() * 1e-6) / 1e9 / HBM_PEAK_GBPS,
        "prefill_call_us": float(pre.mean()), "prefill_call_us_first": float(np.median(first_prefill_us)),
        "prefill_tokens_per_s": w.batch * w.context / (pre.mean() * 1e-6),
        "prefill_algorithmic_bytes": pre_alg,
        "prefill_hbm_gbps": pre_alg / (pre.mean() * 1e-6) / 1e9,
        "prefill_frac_of_hbm_peak": pre_alg / (pre.mean() * 1e-6) / 1e9 / HBM_PEAK_GBPS,
    }
    if name == "c1_mha4_2k":
        res["note"] = "latency-bound (0.9 MB per call): microseconds are the figure, not the bandwidth"
    del caches
    torch.cuda.empty_cache()
    res["read_write_kernel"] = read_write_yardstick(B, torch, w, device)
    res["prefill_frac_of_read_write_kernel"] = res["read_write_kernel"]["gbps"] and res["prefill_hbm_gbps"] / res["read_write_kernel"]["gbps"]
    torch.cuda.empty_cache()
    return res


# ------------------------------------------------------------------ CPU oracle ----

def set_oracle_threads(n: int):
    """Thread count of the OpenMP runtime that the oracle library runs on (the oracle is not changed)."""
    import ctypes
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def oracle_leg(w, ctx_all: int, ctx_one: int | None, n_sink: int = 0, meta: str = "f32", group_bounds=None,
               time_prefill: bool = False) -> dict:
    """Times the CPU oracle (as it stands) on one layer of workload w cut to ctx_all tokens: its own
    prefill from host inputs, then one append and three decodes (min) on all threads; with ctx_one,
    a decode on one thread at that context (min of three).  Times scale linearly in the context."""
    from oracle import skvq_oracle as O
    from paper_2405_06219_amd import synth

    threads = O.num_threads()
    res = {"threads": threads, "context_timed": ctx_all}
    ws = w.scaled(ctx_all)
    k, v = synth.make_kv(ws)
    pk, pv = synth.make_permutations(ws, k[:, :, :4096], v[:, :, :4096])
    ck, cv = synth.make_clip(ws)

    def make(ctx):
        return O.OracleCache(ws.batch, ws.n_q_heads, ws.n_kv_heads, ws.group_size, ws.v_bits, ws.window,
                             ctx - ws.window + 4, pk, pv, ck, cv, n_sink=n_sink, meta=meta, k_bits=ws.k_bits,
                             group_bounds=group_bounds)
    oc = make(ctx_all)
    t0 = time.perf_counter()
    assert oc.prefill(k, v) == 0
    t1 = time.perf_counter()
    if time_prefill:
        res["prefill_us"] = (t1 - t0) * 1e6
        res["prefill_tokens_per_s"] = ws.batch * ctx_all / (t1 - t0)
    q = synth.make_query(ws)
    kn, vn = synth.make_new_token(ws, 0)
    t0 = time.perf_counter()
    assert oc.append(kn, vn) == 0
    res["append_us"] = (time.perf_counter() - t0) * 1e6
    dec = []
    for _ in range(3):
        t0 = time.perf_counter()
        oc.decode(q)
        dec.append((time.perf_counter() - t0) * 1e6)
    res["decode_us"] = min(dec)
    res["decode_us_scaled_to_full_context"] = min(dec) * (w.context / ctx_all)
    if ctx_one:
        one = make(ctx_one)
        assert one.prefill(np.ascontiguousarray(k[:, :, :ctx_one]), np.ascontiguousarray(v[:, :, :ctx_one])) == 0
        set_oracle_threads(1)
        try:
            dec1 = []
            for _ in range(3):
                t0 = time.perf_counter()
                one.decode(q)
                dec1.append((time.perf_counter() - t0) * 1e6)
        finally:
            set_oracle_threads(threads)
        res["one_thread"] = {"context_timed": ctx_one, "decode_us": min(dec1),
                             "decode_us_scaled_to_full_context": min(dec1) * (w.context / ctx_one)}
    return res


def bounded_context(w, token_heads: int) -> int:
    """Largest power-of-two context (at most w.context) with about `token_heads` (sequence, head, token)
    triples per decode: bounds the oracle's time."""
    ctx = w.context
    while ctx > 1024 and ctx * w.batch * w.n_q_heads > token_heads:
        ctx //= 2
    return ctx


# ------------------------------------------------------------------ profiler workloads ----

def probe(args, w, bounds, device) -> int:
    import torch
    from paper_2405_06219_amd import binding as B
    from paper_2405_06219_amd import synth

    if args.probe == "decode":
        # a few decode calls (first skvq_decode_attention alone, then skvq_append_decode_attention), then a
        # plain 256 MiB device-to-device copy: what FETCH_SIZE / WRITE_SIZE read for it scales the counters
        n_layers = args.layers if args.layers else 4
        caches = build_layers(w, n_layers, 8, device, args.sink, args.meta, bounds)[0]
        q = torch.randn((n_layers, w.batch, w.n_q_heads, D), device=device).to(torch.float16)
        out = torch.empty((n_layers, w.batch, w.n_q_heads, D), dtype=torch.float32, device=device)
        kn = torch.randn((n_layers, w.batch, w.n_kv_heads, D), device=device).to(torch.float16)
        vn = torch.randn((n_layers, w.batch, w.n_kv_heads, D), device=device).to(torch.float16)
        for _ in range(3):
            for i, c in enumerate(caches):
                c.skvq_decode_attention(q[i], out_f32=out[i])
        for _ in range(3):
            for i, c in enumerate(caches):
                c.skvq_append_decode_attention(kn[i], vn[i], q[i], out_f32=out[i])
        torch.cuda.synchronize()
        src = torch.ones(256 << 20, dtype=torch.uint8, device=device)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(f"probe decode: {w.name}, {n_layers} layers, 3 x skvq_decode_attention then 3 x "
              f"skvq_append_decode_attention per layer, then 3 copies of 268435456 bytes; "
              f"decode algorithmic bytes per call: {algorithmic_bytes_decode(w, w.context, args.sink, args.meta)}; "
              f"prefill algorithmic bytes per call: {algorithmic_bytes_prefill(w, args.meta)}; "
              f"source_fingerprint: {source_fingerprint()}")
        return 0
    if args.probe == "prefill":
        # skvq_prefill_quantize of every layer, the calls back to back, three rounds
        n_layers = args.layers if args.layers else 8
        caches, _, first_us, sources = build_layers(w, n_layers, 8, device, args.sink, args.meta, bounds, keep_sources=True)

        def prefill_all():
            for c, (k, v) in zip(caches, sources):
                c.skvq_prefill_quantize(k, v)
        us = timed_us(prefill_all, n_layers, 3, warm=0)
        by = algorithmic_bytes_prefill(w, args.meta)
        print(f"probe prefill: {w.name}, {n_layers} layers: first call of each layer (own pair of events) {np.median(first_us):.2f} us, "
              f"then 3 rounds back to back {us.mean():.2f} us per call ({by / us.mean() / 1e3:.0f} GB/s = "
              f"{100 * by / us.mean() / 1e3 / HBM_PEAK_GBPS:.1f} % of {HBM_PEAK_GBPS:.0f} GB/s); algorithmic bytes per call {by}; "
              f"source_fingerprint: {source_fingerprint()}")
        return 0
    if args.probe == "prefill-attention":
        T = w.context if args.context else 32768
        perm = np.tile(np.arange(D, dtype=np.int32), (w.n_kv_heads, 1))
        one = np.ones((w.n_kv_heads, 1), np.float32)
        cache = B.SkvqCache(1, w.n_q_heads, w.n_kv_heads, 128, 1.5, 8, 8, perm, perm, one, one, device=device)
        gen = torch.Generator(device=device)
        gen.manual_seed(7)
        q = torch.randn((1, w.n_q_heads, T, D), generator=gen, device=device).to(torch.float16)
        k = torch.randn((1, w.n_kv_heads, T, D), generator=gen, device=device).to(torch.float16)
        v = torch.randn((1, w.n_kv_heads, T, D), generator=gen, device=device).to(torch.float16)
        out = torch.empty((1, w.n_q_heads, T, D), dtype=torch.float32, device=device)
        us = timed_us(lambda: cache.skvq_prefill_attention(q, k, v, out_f32=out), 1, 5)
        flops = 4.0 * D * w.n_q_heads * T * (T + 1) / 2
        print(f"probe prefill-attention: {w.n_q_heads} q / {w.n_kv_heads} kv heads, {T} tokens: {us.mean() / 1e3:.3f} ms per "
              f"call, {flops / us.mean() / 1e6:.1f} TFLOP/s ({100 * flops / (us.mean() * 1e-6) / MFMA_F16_PEAK_FLOPS:.1f} % of "
              f"2.5 PFLOP/s); source_fingerprint: {source_fingerprint()}")
        return 0
    if args.probe == "read":
        # the read-only kernel over slices of the decode call's size, rotating through 2.5 GB (cold HBM),
        # and over the whole 2.5 GB at once
        total = 2560 << 20
        buf = torch.ones(total, dtype=torch.uint8, device=device)
        sink = torch.zeros(4, dtype=torch.uint8, device=device)
        for label, nbytes in (("decode call of " + w.name, algorithmic_bytes_decode(w, w.context) & ~0xFFF),
                              ("2.5 GB", total)):
            n_slices = max(total // nbytes, 1)
            slices = [buf[i * nbytes:(i + 1) * nbytes] for i in range(n_slices)]

            def sweep():
                for s_ in slices:
                    B.skvq_read_yardstick(s_, sink)
            us = timed_us(sweep, n_slices, 5)
            print(f"probe read: {nbytes} bytes ({label}), {n_slices} slices back to back: {us.mean():.2f} us per launch "
                  f"(min {us.min():.2f}), {nbytes / us.mean() / 1e3:.0f} GB/s = {100 * nbytes / us.mean() / 1e3 / HBM_PEAK_GBPS:.1f} % "
                  f"of {HBM_PEAK_GBPS:.0f} GB/s")
        del buf, slices
        torch.cuda.empty_cache()
        # the read/write kernel on the prefill call's traffic, at this workload and at the batch-16 one
        for wl in (w, synth.WORKLOADS["c5_batch16_32k"]):
            r = read_write_yardstick(B, torch, wl, device)
            print(f"probe read/write: prefill call of {wl.name}: {r['read_bytes']} bytes read + {r['write_bytes']} written, "
                  f"back to back: {r['us_per_launch']:.2f} us per launch, {r['gbps']:.0f} GB/s = "
                  f"{100 * r['frac_of_hbm_peak']:.1f} % of {HBM_PEAK_GBPS:.0f} GB/s")
        return 0
    print(f"unknown probe {args.probe}", file=sys.stderr)
    return 2


# ------------------------------------------------------------------ main ----

def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--layers", type=int, default=0, help="layer caches rotated (default 32; probes: 4)")
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--context", type=int, default=0, help="override the workload's context (tests)")
    ap.add_argument("--sink", type=int, default=0,
                    help="attention sinks: the first N tokens stay fp16 (the headline workload has none)")
    ap.add_argument("--meta", choices=sorted(META_BYTES), default="f32",
                    help="storage of (scale, zero); the headline workload keeps them in fp32")
    ap.add_argument("--k-bits", type=float, choices=[2.0, 3.0, 4.0], default=0.0,
                    help="override the workload's key width (the headline workload has 2-bit keys)")
    ap.add_argument("--v-bits", type=float, choices=[1.5, 2.0, 3.0, 4.0], default=0.0,
                    help="override the workload's value width (the headline workload has 1.5-bit values)")
    ap.add_argument("--group-size", type=int, choices=[32, 64, 128], default=0,
                    help="override the workload's (average) group size (the headline workload has 128)")
    ap.add_argument("--group-bounds", default="",
                    help="unequal groups: comma-separated boundaries, 128/group_size + 1 multiples of 16 from 0 to 128")
    ap.add_argument("--two-calls", action="store_true",
                    help="time skvq_quantize_append + skvq_decode_attention per layer instead of the one call "
                         "that does both (skvq_append_decode_attention)")
    ap.add_argument("--configs", choices=["all", "none"], default="all",
                    help="also measure the other baseline configurations (default, when the headline workload runs "
                         "in its own format)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--probe", default="", help="run a profiler workload instead: decode | prefill | prefill-attention | read")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import torch
    from paper_2405_06219_amd import binding as B
    from paper_2405_06219_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    B.lib()  # fail loudly if the HIP library is missing
    device = torch.device("cuda:0")
    torch.cuda.set_device(device)
    w = synth.WORKLOADS[args.workload]
    if args.context:
        w = w.scaled(args.context)
    headline_format = not args.k_bits and not args.v_bits and not args.group_size and not args.group_bounds
    if args.group_size:
        w = dataclasses.replace(w, group_size=args.group_size)
    bounds = [int(x) for x in args.group_bounds.split(",")] if args.group_bounds else None
    if args.k_bits:
        w = dataclasses.replace(w, k_bits=args.k_bits)
    if args.v_bits:
        w = dataclasses.replace(w, v_bits=args.v_bits)
    if args.probe:
        return probe(args, w, bounds, device)
    n_steps, n_warm, n_layers = args.steps, args.warmup, args.layers if args.layers else 32
    headroom = n_warm + 3 * n_steps + 9
    as_baseline = (headline_format and w.context == synth.WORKLOADS[w.name].context and not args.sink
                   and args.meta == "f32")

    caches, (sk_d, sv_d), prefill_us, sources = build_layers(w, n_layers, headroom, device, args.sink, args.meta, bounds,
                                                             keep_sources=True)
    # prefill again with the layers' calls back to back: one pair of events around all of them
    def prefill_all():
        for c, (k, v) in zip(caches, sources):
            c.skvq_prefill_quantize(k, v)
    prefill_b2b = timed_us(prefill_all, n_layers, 3, warm=0)
    del sources
    torch.cuda.empty_cache()
    prefill_call_us = float(prefill_b2b.mean())
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed)
    total = n_warm + 3 * n_steps + 1
    # per (step, layer) inputs, resident before the timed region
    q_all = torch.randn((total, n_layers, w.batch, w.n_q_heads, D), generator=gen, device=device).to(torch.float16)
    kn_all = (torch.randn((total, n_layers, w.batch, w.n_kv_heads, D), generator=gen, device=device)
              * sk_d[:, :, 0]).to(torch.float16)
    vn_all = (torch.randn((total, n_layers, w.batch, w.n_kv_heads, D), generator=gen, device=device)
              * sv_d[:, :, 0]).to(torch.float16)
    out = torch.empty((n_layers, w.batch, w.n_q_heads, D), dtype=torch.float32, device=device)

    # The host side of a call (tensor views, argument checks, the ctypes call) costs about 10 us, the call
    # itself 25 us on the GPU: the views are taken before the timed region, the stream is passed along and
    # the collector is off inside it, so that a pause of the interpreter does not show up as GPU time.
    stream = torch.cuda.current_stream()
    views = [[(kn_all[i, layer], vn_all[i, layer], q_all[i, layer], out[layer]) for layer in range(n_layers)]
             for i in range(total)]

    def step_one_call(i):
        for c, (kn, vn, q, o) in zip(caches, views[i]):
            c.skvq_append_decode_attention(kn, vn, q, out_f32=o, stream=stream)

    def step_two_calls(i):
        for c, (kn, vn, q, o) in zip(caches, views[i]):
            c.skvq_quantize_append(kn, vn, stream=stream)
            c.skvq_decode_attention(q, out_f32=o, stream=stream)

    step, other_step = (step_two_calls, step_one_call) if args.two_calls else (step_one_call, step_two_calls)
    # (an idle GPU takes about ten milliseconds of work to come back to its clocks: nothing slow may sit
    # between the warm-up steps and the timed ones)
    gc.collect()
    gc.disable()
    # (decode calls that change nothing, about 15 ms of them, whatever the warm-up count asked for)
    for _ in range(20):
        for c, (kn, vn, q, o) in zip(caches, views[0]):
            c.skvq_decode_attention(q, out_f32=o, stream=stream)
    i = 0
    for _ in range(n_warm):
        step(i)
        i += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n_steps):
        step(i)
        i += 1
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gc.enable()
    ms_per_step = (t1 - t0) * 1e3 / n_steps
    # the same steps the other way, for comparison
    t0 = time.perf_counter()
    for _ in range(n_steps):
        other_step(i)
        i += 1
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    other_ms_per_step = (t1 - t0) * 1e3 / n_steps

    # roofline pass: the decode launches of all layers back to back between one pair of HIP events;
    # average launch duration = elapsed / layers.  With two calls per layer the appends of all layers go
    # first, untimed.
    dec_us = []
    for _ in range(n_steps):
        if args.two_calls:
            for layer, c in enumerate(caches):
                c.skvq_quantize_append(kn_all[i, layer], vn_all[i, layer])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        if args.two_calls:
            for layer, c in enumerate(caches):
                c.skvq_decode_attention(q_all[i, layer], out_f32=out[layer])
        else:
            step_one_call(i)
        e1.record()
        torch.cuda.synchronize()
        dec_us.append(e0.elapsed_time(e1) * 1e3 / n_layers)
        i += 1
    dec_us = np.array(dec_us)
    dec_avg_us = float(dec_us.mean())
    n_tokens_roof = w.context + n_warm + 2 * n_steps + n_steps // 2
    alg_bytes = algorithmic_bytes_decode(w, n_tokens_roof, args.sink, args.meta)
    achieved = alg_bytes / (dec_avg_us * 1e-6) / 1e9

    # the read-only kernel over slices of the same size (what a kernel that only has to read that much takes here)
    read_buf = torch.ones(max(n_layers, 8) * (alg_bytes & ~0xFFF), dtype=torch.uint8, device=device)
    read_sink = torch.zeros(4, dtype=torch.uint8, device=device)
    slice_bytes = alg_bytes & ~0xFFF
    slices = [read_buf[j * slice_bytes:(j + 1) * slice_bytes] for j in range(max(n_layers, 8))]

    def read_sweep():
        for s_ in slices:
            B.skvq_read_yardstick(s_, read_sink)
    read_us = float(timed_us(read_sweep, len(slices), 5).mean())
    del read_buf, slices
    torch.cuda.empty_cache()
    # the read/write kernel on the prefill call's traffic
    rw = read_write_yardstick(B, torch, w, device)
    torch.cuda.empty_cache()

    # the prompt's own causal attention (skvq_prefill_attention) at 16k tokens of the same head
    # layout: a dense contraction, reported against the fp16 matrix-core peak
    pa = None
    if w.batch == 1:
        pa_T = min(16384, w.context)
        pa_q = torch.randn((1, w.n_q_heads, pa_T, D), generator=gen, device=device).to(torch.float16)
        pa_k = (torch.randn((1, w.n_kv_heads, pa_T, D), generator=gen, device=device) * sk_d).to(torch.float16)
        pa_v = (torch.randn((1, w.n_kv_heads, pa_T, D), generator=gen, device=device) * sv_d).to(torch.float16)
        pa_out = torch.empty((1, w.n_q_heads, pa_T, D), dtype=torch.float32, device=device)
        pa_us = timed_us(lambda: caches[0].skvq_prefill_attention(pa_q, pa_k, pa_v, out_f32=pa_out), 1, 3)
        pa_flops = 4.0 * D * w.n_q_heads * pa_T * (pa_T + 1) / 2
        pa = {"tokens": pa_T, "ms_per_call": float(pa_us.mean()) / 1e3,
              "tflops": pa_flops / (pa_us.mean() * 1e-6) / 1e12,
              "frac_of_mfma_peak": pa_flops / (pa_us.mean() * 1e-6) / MFMA_F16_PEAK_FLOPS,
              "arithmetic": "f16 matrix-core operands (weights as a high and a low f16 part), f32 accumulation"}
        del pa_q, pa_k, pa_v, pa_out

    # several query tokens per call (skvq_decode_attention_multi): the layers' calls back to back
    multi_us = {}
    for n_new in MULTI_TOKENS:
        qm = torch.randn((n_layers, w.batch, n_new, w.n_q_heads, D), generator=gen, device=device).to(torch.float16)
        om = torch.empty((n_layers, w.batch, n_new, w.n_q_heads, D), dtype=torch.float32, device=device)

        def multi():
            for layer, c in enumerate(caches):
                c.skvq_decode_attention_multi(qm[layer], out_f32=om[layer])
        multi_us[str(n_new)] = float(timed_us(multi, n_layers, 3).mean())
        del qm, om

    # append alone (launch-latency bound, reported for completeness)
    def append_all():
        for layer, c in enumerate(caches):
            c.skvq_quantize_append(kn_all[i, layer], vn_all[i, layer])
    append_us = float(timed_us(append_all, n_layers, 3, warm=0).min())  # (the first round also loads the kernel)

    pre_alg = algorithmic_bytes_prefill(w, args.meta)
    facts = profile_facts(w.name) if as_baseline else {}
    fp = source_fingerprint()
    pmc, ktr = facts.get("pmc", {}), facts.get("kernel_trace", {})
    traffic = int(pmc["traffic_bytes_per_call"]) if pmc.get("source_fingerprint") == fp and "traffic_bytes_per_call" in pmc else None
    kernel_avg_us = float(ktr["kernel_avg_us"]) if ktr.get("source_fingerprint") == fp and "kernel_avg_us" in ktr else None
    kernel_name = (f"decode_mfma_kernel<R={min(w.n_q_heads // w.n_kv_heads, 4)}, K levels {int(2 ** w.k_bits)}, "
                   f"V levels {3 if w.v_bits == 1.5 else int(2 ** w.v_bits)}, meta {args.meta}, "
                   f"{D // w.group_size} group(s)> + merge_kernel")
    result = {
        "metric": "decode-attention us/token at 128k ctx" if w.context == 131072 else f"decode-attention us/token at {w.context} ctx",
        "value": ms_per_step * 1e3,
        "unit": "us/token",
        "n_gpus": 1,
        "steps": n_steps,
        "warmup": n_warm,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 MFMA operands, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": w.name, "layers": n_layers, "batch": w.batch, "n_q_heads": w.n_q_heads,
                   "n_kv_heads": w.n_kv_heads, "head_dim": D, "context": w.context, "k_bits": w.k_bits,
                   "v_bits": w.v_bits, "group_size": w.group_size, "window": w.window, "n_sink": args.sink, "meta": args.meta,
                   "group_bounds": bounds,
                   "step": ("per layer: skvq_quantize_append + skvq_decode_attention" if args.two_calls else
                            "per layer: skvq_append_decode_attention (append and attention in one launch + merge)")},
        "us_per_layer": ms_per_step * 1e3 / n_layers,
        ("one_call_us_per_token" if args.two_calls else "two_calls_us_per_token"): other_ms_per_step * 1e3,
        "decode_call_us": dec_avg_us,
        "decode_call_us_min": float(dec_us.min()),
        "append_call_us": append_us,
        "decode_multi_call_us": multi_us,
        "prefill_call_us": prefill_call_us,
        "prefill_call_us_single_with_events": float(np.median(prefill_us)),
        "prefill_tokens_per_s": w.batch * w.context / (prefill_call_us * 1e-6),
        "prefill_hbm_gbps": pre_alg / (prefill_call_us * 1e-6) / 1e9,
        "prefill_frac_of_hbm_peak": pre_alg / (prefill_call_us * 1e-6) / 1e9 / HBM_PEAK_GBPS,
        "prefill_frac_of_read_write_kernel": pre_alg / (prefill_call_us * 1e-6) / 1e9 / rw["gbps"],
        "read_write_kernel": rw,
        "prefill_attention": pa,
        "effective_hbm_gbps": achieved,
        "pct_of_hbm_peak": 100.0 * achieved / HBM_PEAK_GBPS,
        "read_only_kernel": {"bytes": slice_bytes, "us_per_launch": read_us, "gbps": slice_bytes / read_us / 1e3,
                             "frac_of_hbm_peak": slice_bytes / read_us / 1e3 / HBM_PEAK_GBPS,
                             "what": "skvq_read_yardstick over slices of the decode call's size, back to back"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": traffic,
                     "traffic_source": ("profiles/decode_%s_pmc.txt (same kernel sources)" % w.name if traffic is not None else
                                        "no counter summary for these kernel sources"),
                     "kernel": kernel_name,
                     "launch": "one call = chunk kernel + merge kernel; duration from HIP events around the layers' calls back to back",
                     "bytes_per_launch": alg_bytes,
                     "avg_launch_us": dec_avg_us,
                     "frac_call": achieved / HBM_PEAK_GBPS,
                     "frac_chunk_kernel_profile": (alg_bytes / (kernel_avg_us * 1e-6) / 1e9 / HBM_PEAK_GBPS
                                                   if kernel_avg_us else None),
                     "chunk_kernel_avg_us_profile": kernel_avg_us,
                     "frac_of_read_only_kernel": read_us / dec_avg_us},
    }
    del caches, q_all, kn_all, vn_all
    torch.cuda.empty_cache()

    if args.configs == "all" and as_baseline and w.name == HEADLINE:
        result["configs"] = {}
        for name in OTHER_CONFIGS:
            result["configs"][name] = measure_config(name, device, n_steps)

    if not args.no_cpu_baseline:
        # the oracle: all threads at the full context (bounded: shrunk if a decode would take too long), one
        # thread at a shorter one; min of three decodes each
        ctx = bounded_context(w, 6_000_000)
        cb = oracle_leg(w, ctx, min(ctx, bounded_context(w, 600_000)), args.sink, args.meta, bounds)
        per_layer_us = (cb["append_us"] + cb["decode_us"]) * (w.context / ctx)
        result["cpu_baseline"] = {
            "value": per_layer_us * n_layers, "unit": "us/token", "cores": cb["threads"], "kind": "oracle",
            "sample": (f"1 of {n_layers} layers (append + decode, min of 3 decodes) at context {ctx}"
                       f", scaled to {w.context} tokens and x{n_layers} layers"),
            "decode_us_timed": cb["decode_us"], "append_us_timed": cb["append_us"],
            "one_thread": cb.get("one_thread")}
        if "configs" in result:
            from paper_2405_06219_amd import synth as S
            for name in OTHER_CONFIGS:
                wc = S.WORKLOADS[name]
                full = name in ("c1_mha4_2k", "c2_llama7b_32k")
                ctx_c = wc.context if full else bounded_context(wc, 2_000_000)
                leg = oracle_leg(wc, ctx_c, min(ctx_c, bounded_context(wc, 600_000)) if full else None,
                                 time_prefill=(name == "c5_batch16_32k"))
                leg["kind"] = "oracle"
                leg["sample"] = (f"one layer, one decode step (min of 3) at context {ctx_c} of {wc.context}"
                                 + ("" if full else ", times scale linearly in the context"))
                result["configs"][name]["cpu_baseline"] = leg
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
