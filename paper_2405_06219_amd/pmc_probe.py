"""Workload for hardware-counter runs: a few decode steps on the benchmark's layer shape (first
skvq_decode_attention alone, then skvq_append_decode_attention) and a plain device-to-device
copy of known size (the yardstick that FETCH_SIZE / WRITE_SIZE are scaled by).  Run under
`rocprofv3 --pmc FETCH_SIZE` (and again with WRITE_SIZE):

    python3 paper_2405_06219_amd/pmc_probe.py [workload] [layers] [meta format] [sinks]

The chunk kernel's dispatches come in two sets of 3 x layers: the first without, the second with
the append.
"""
from __future__ import annotations

import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main() -> int:
    import bench
    from paper_2405_06219_amd import synth

    name = sys.argv[1] if len(sys.argv) > 1 else "c3_mistral7b_128k"
    n_layers = int(sys.argv[2]) if len(sys.argv) > 2 else 4
    dev = torch.device("cuda:0")
    w = synth.WORKLOADS[name]
    meta = sys.argv[3] if len(sys.argv) > 3 else "f32"
    n_sink = int(sys.argv[4]) if len(sys.argv) > 4 else 0
    caches = bench.build_layers(w, n_layers, 8, dev, n_sink, meta)[0]
    q = torch.randn((n_layers, w.batch, w.n_q_heads, 128), device=dev).to(torch.float16)
    out = torch.empty((n_layers, w.batch, w.n_q_heads, 128), dtype=torch.float32, device=dev)
    for _ in range(3):
        for i, c in enumerate(caches):
            c.skvq_decode_attention(q[i], out_f32=out[i])
    kn = torch.randn((n_layers, w.batch, w.n_kv_heads, 128), device=dev).to(torch.float16)
    vn = torch.randn((n_layers, w.batch, w.n_kv_heads, 128), device=dev).to(torch.float16)
    for _ in range(3):
        for i, c in enumerate(caches):
            c.skvq_append_decode_attention(kn[i], vn[i], q[i], out_f32=out[i])
    torch.cuda.synchronize()
    # yardstick: copy 256 MiB (reads 268435456 bytes, writes 268435456 bytes)
    src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    print("decode algorithmic bytes per call:", bench.algorithmic_bytes_decode(w, w.context, n_sink, meta))
    return 0


if __name__ == "__main__":
    sys.exit(main())
