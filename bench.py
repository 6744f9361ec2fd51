#!/usr/bin/env python3
"""Benchmark of the SKVQ hot path on one MI355X.

A step is one generated token of a 7B-shaped model: for each of `--layers` attention layers
(each with its own cache, so that no layer's data is still in the 256 MB Infinity Cache when
its turn comes again) the token leaving the fp16 window is quantized and the new query attends
over the whole cache: one skvq_append_decode_attention call per layer (with --two-calls:
skvq_quantize_append, then skvq_decode_attention; the other way is timed too and reported
beside).  Inputs are seeded synthetic tensors already resident in HBM.

Prints ONE JSON line.  `value` is microseconds per token (all layers); `roofline` prices the
algorithmic bytes of one layer's attention call against the 8 TB/s HBM peak, its duration
measured with HIP events around the layers' calls issued back to back; `cpu_baseline` is the
CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
D = 128
# HBM bytes per attention call (one call with the append inside / skvq_decode_attention alone)
# measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (chunk kernel + merge kernel, counters
# scaled by a plain copy of known size); see profiles/decode_c3_mistral7b_128k_pmc.txt.  Only
# workloads that were measured have an entry.
MEASURED_TRAFFIC_BYTES = {"c3_mistral7b_128k": (78037 * 1024, 78007 * 1024)}


META_BYTES = {"f32": 4, "f16": 2, "e4m3": 1}
MULTI_TOKENS = (2, 4)  # query tokens per call timed for skvq_decode_attention_multi


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


def build_layers(w, n_layers: int, headroom: int, device, n_sink: int = 0, meta: str = "f32", group_bounds=None):
    """Per layer: a cache prefilled with w.context seeded synthetic tokens.  Returns the caches,
    the K/V channel scales on the device, and each prefill call's duration (HIP events, us)."""
    import torch
    from paper_2405_06219_amd import binding as B
    from paper_2405_06219_amd import synth

    sk, sv = synth.channel_scales(w)
    sk_d = torch.from_numpy(sk).to(device)[None, :, None, :]
    sv_d = torch.from_numpy(sv).to(device)[None, :, None, :]
    ck, cv = synth.make_clip(w)
    caches = []
    prefill_us = []
    for layer in range(n_layers):
        # seeded synthetic K/V and the reorder index from their channel ranges (offline calibration stand-in)
        k, v, pk, pv = synth.make_kv_device(w, device, stream=layer)
        c = B.SkvqCache(w.batch, w.n_q_heads, w.n_kv_heads, w.group_size, w.v_bits, w.window,
                        w.context - w.window + headroom, pk, pv, ck, cv, device=device, n_sink=n_sink,
                        meta=meta, k_bits=w.k_bits, group_bounds=group_bounds, max_new_tokens=MULTI_TOKENS[-1])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        c.skvq_prefill_quantize(k, v)
        e1.record()
        torch.cuda.synchronize()
        prefill_us.append(e0.elapsed_time(e1) * 1e3)
        del k, v
        caches.append(c)
    return caches, (sk_d, sv_d), prefill_us


def cpu_baseline(w, n_sink: int = 0, meta: str = "f32", group_bounds=None, seconds_budget: float = 25.0):
    """Times the CPU oracle (as it stands) on one layer of the same workload: its own prefill
    from host inputs (untimed), then one append + one decode (timed)."""
    from oracle import skvq_oracle as O
    from paper_2405_06219_amd import synth

    # bound the sample: shrink the context until the oracle's decode fits the budget
    ctx = w.context
    per_token_ns = 1100.0 * w.n_q_heads * w.batch / max(O.num_threads(), 1)
    while ctx > 4096 and ctx * per_token_ns * 1e-9 > seconds_budget / 3:
        ctx //= 2
    ws = w.scaled(ctx)
    k, v = synth.make_kv(ws)
    pk, pv = synth.make_permutations(ws, k[:, :, :4096], v[:, :, :4096])
    ck, cv = synth.make_clip(ws)
    oc = O.OracleCache(ws.batch, ws.n_q_heads, ws.n_kv_heads, ws.group_size, ws.v_bits, ws.window,
                       ctx - ws.window + 4, pk, pv, ck, cv, n_sink=n_sink, meta=meta, k_bits=ws.k_bits,
                       group_bounds=group_bounds)
    assert oc.prefill(k, v) == 0
    q = synth.make_query(ws)
    kn, vn = synth.make_new_token(ws, 0)
    t0 = time.perf_counter()
    assert oc.append(kn, vn) == 0
    t1 = time.perf_counter()
    oc.decode(q)
    t2 = time.perf_counter()
    per_layer_us = (t2 - t0) * 1e6 * (w.context / ctx)
    return {"per_layer_us": per_layer_us, "append_us": (t1 - t0) * 1e6, "decode_us": (t2 - t1) * 1e6,
            "context_timed": ctx, "threads": O.num_threads()}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--workload", default="c3_mistral7b_128k")
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
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    n_steps, n_warm, n_layers = args.steps, args.warmup, args.layers
    headroom = n_warm + 3 * n_steps + 9

    caches, (sk_d, sv_d), prefill_us = build_layers(w, n_layers, headroom, device, args.sink, args.meta, bounds)
    prefill_med_us = float(np.median(prefill_us))
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

    def step_one_call(i):
        for layer, c in enumerate(caches):
            c.skvq_append_decode_attention(kn_all[i, layer], vn_all[i, layer], q_all[i, layer], out_f32=out[layer])

    def step_two_calls(i):
        for layer, c in enumerate(caches):
            c.skvq_quantize_append(kn_all[i, layer], vn_all[i, layer])
            c.skvq_decode_attention(q_all[i, layer], out_f32=out[layer])

    step, other_step = (step_two_calls, step_one_call) if args.two_calls else (step_one_call, step_two_calls)
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
    ms_per_step = (t1 - t0) * 1e3 / n_steps
    n_tokens_mid = w.context + n_warm + n_steps // 2
    # the same steps the other way, for comparison
    t0 = time.perf_counter()
    for _ in range(n_steps):
        other_step(i)
        i += 1
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    other_ms_per_step = (t1 - t0) * 1e3 / n_steps

    # roofline pass: the decode launches of all layers back to back between one pair of HIP events
    # (an event pair around every single call adds about 2 us to each); average launch duration =
    # elapsed / layers.  With two calls per layer the appends of all layers go first, untimed.
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

    # the prompt's own causal attention (skvq_prefill_attention) at 16k tokens of the same head
    # layout: a dense contraction, reported against the fp16 matrix-core peak
    pa_T = min(16384, w.context)
    pa_q = torch.randn((1, w.n_q_heads, pa_T, D), generator=gen, device=device).to(torch.float16)
    pa_k = (torch.randn((1, w.n_kv_heads, pa_T, D), generator=gen, device=device) * sk_d).to(torch.float16)
    pa_v = (torch.randn((1, w.n_kv_heads, pa_T, D), generator=gen, device=device) * sv_d).to(torch.float16)
    pa_out = torch.empty((1, w.n_q_heads, pa_T, D), dtype=torch.float32, device=device)
    pa_cache = caches[0] if w.batch == 1 else None
    pa_ms = None
    if pa_cache is not None:
        pa_cache.skvq_prefill_attention(pa_q, pa_k, pa_v, out_f32=pa_out)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            pa_cache.skvq_prefill_attention(pa_q, pa_k, pa_v, out_f32=pa_out)
        e1.record()
        torch.cuda.synchronize()
        pa_ms = e0.elapsed_time(e1) / 3
    del pa_q, pa_k, pa_v, pa_out

    # several query tokens per call (skvq_decode_attention_multi): the layers' calls back to back
    multi_us = {}
    for n_new in MULTI_TOKENS:
        qm = torch.randn((n_layers, w.batch, n_new, w.n_q_heads, D), generator=gen, device=device).to(torch.float16)
        om = torch.empty((n_layers, w.batch, n_new, w.n_q_heads, D), dtype=torch.float32, device=device)
        for rep in range(4):  # the first repetition warms up
            if rep == 1:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
            for layer, c in enumerate(caches):
                c.skvq_decode_attention_multi(qm[layer], out_f32=om[layer])
        e1.record()
        torch.cuda.synchronize()
        multi_us[str(n_new)] = e0.elapsed_time(e1) * 1e3 / (3 * n_layers)
        del qm, om

    # append alone (launch-latency bound, reported for completeness): one pair of HIP events
    # around the layers' calls issued back to back
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for layer, c in enumerate(caches):
        c.skvq_quantize_append(kn_all[i, layer], vn_all[i, layer])
    e1.record()
    torch.cuda.synchronize()
    append_us = e0.elapsed_time(e1) * 1e3 / n_layers

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
        "dtype": "f32",
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
        "prefill_call_us": prefill_med_us,
        "prefill_tokens_per_s": w.batch * w.context / (prefill_med_us * 1e-6),
        "prefill_hbm_gbps": (w.batch * w.n_kv_heads * (w.context * 2 * D * 2 + max(w.context - w.window, 0)
                                                     * (code_bytes_per_row(w)
                                                        + 4 * META_BYTES[args.meta] * (D // w.group_size)))
                             / (prefill_med_us * 1e-6) / 1e9),
        "prefill_attention": (None if pa_ms is None else {
            "tokens": pa_T, "ms_per_call": pa_ms,
            "tflops": 4.0 * D * w.n_q_heads * pa_T * (pa_T + 1) / 2 / (pa_ms * 1e-3) / 1e12,
            "frac_of_mfma_peak": 4.0 * D * w.n_q_heads * pa_T * (pa_T + 1) / 2 / (pa_ms * 1e-3) / 2.5e15}),
        "effective_hbm_gbps": achieved,
        "pct_of_hbm_peak": 100.0 * achieved / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": (MEASURED_TRAFFIC_BYTES[w.name][1 if args.two_calls else 0]
                                 if w.name in MEASURED_TRAFFIC_BYTES and w.context == synth.WORKLOADS[w.name].context and not args.sink
                                 and args.meta == "f32" and headline_format else None),
                     "kernel": "skvq_decode_attention" if args.two_calls else "skvq_append_decode_attention",
                     "bytes_per_launch": alg_bytes,
                     "avg_launch_us": dec_avg_us},
    }
    if not args.no_cpu_baseline:
        cb = cpu_baseline(w, args.sink, args.meta, bounds)
        result["cpu_baseline"] = {
            "value": cb["per_layer_us"] * n_layers, "unit": "us/token", "cores": cb["threads"], "kind": "oracle",
            "sample": (f"1 of {n_layers} layers (append + decode) at context {cb['context_timed']}"
                       f", scaled to {w.context} tokens and x{n_layers} layers"),
            "decode_us_timed": cb["decode_us"], "append_us_timed": cb["append_us"]}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
