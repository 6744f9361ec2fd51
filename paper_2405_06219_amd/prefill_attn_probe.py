"""Workload for profiler runs of skvq_prefill_attention: a few calls at one shape.
`python -m paper_2405_06219_amd.prefill_attn_probe [batch] [q_heads] [kv_heads] [tokens] [calls]`"""
from __future__ import annotations

import sys

import numpy as np
import torch

from paper_2405_06219_amd import binding as B

D = 128


def main() -> int:
    b, hq, hk, T, calls = (int(x) for x in (sys.argv[1:6] + ["1", "32", "8", "32768", "5"][len(sys.argv) - 1:]))
    dev = torch.device("cuda:0")
    perm = np.tile(np.arange(D, dtype=np.int32), (hk, 1))
    one = np.ones((hk, 1), np.float32)
    cache = B.SkvqCache(b, hq, hk, 128, 1.5, 8, 8, perm, perm, one, one, device=dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    q = torch.randn((b, hq, T, D), generator=gen, device=dev).to(torch.float16)
    k = torch.randn((b, hk, T, D), generator=gen, device=dev).to(torch.float16)
    v = torch.randn((b, hk, T, D), generator=gen, device=dev).to(torch.float16)
    out = torch.empty((b, hq, T, D), dtype=torch.float32, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    cache.skvq_prefill_attention(q, k, v, out_f32=out)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(calls):
        cache.skvq_prefill_attention(q, k, v, out_f32=out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / calls
    flops = 4.0 * D * hq * b * T * (T + 1) / 2      # causal: QK^T and PV, 2 flops per multiply-add
    print(f"skvq_prefill_attention B{b} Hq{hq} Hk{hk} T{T}: {ms:.3f} ms per call, {flops / ms / 1e9:.1f} TFLOP/s "
          f"({100 * flops / ms / 1e9 / 2500:.1f} % of 2.5 PFLOP/s)")
    return 0


if __name__ == "__main__":
    sys.exit(main())
