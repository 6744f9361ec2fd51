"""Seeded synthetic inputs shaped like the paper's long-context decode workloads.

This module only draws random tensors and sorts channels; it holds none of the
method's arithmetic (no quantizer, no packing, no attention).  Both the CPU
oracle and the HIP path are fed from here so that they see identical bits.

The paper evaluates on Llama-2-7B / Mistral-7B key/value activations whose
channels differ widely in magnitude (Section 3.1, first paragraphs).  Model
weights and datasets are not available, so the stand-in is: i.i.d. normal
values with a per-channel magnitude profile, and a reorder permutation that
sorts channels by a per-channel statistic (the paper clusters channels by
their statistics; sorting by range is the one-dimensional analogue).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

HEAD_DIM = 128


@dataclass(frozen=True)
class Workload:
    """One attention layer's cache shape and quantization setting."""

    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    context: int            # tokens already in the cache when decode starts
    v_bits: float           # 4.0, 3.0, 2.0 or 1.5
    group_size: int = 128
    clip: float = 0.95
    window: int = 128
    channel_profile: str = "loguniform"   # or "outlier4"
    perm_stat: str = "range"              # or "absmax"
    seed: int = 1000
    head_dim: int = HEAD_DIM
    k_bits: float = 2.0     # 2.0, 3.0 or 4.0 (3.0 only with 3-bit values)

    def scaled(self, context: int, batch: int | None = None) -> "Workload":
        """Same layer shape at another context length (for quick tests)."""
        return replace(self, context=context, batch=self.batch if batch is None else batch)


# The five configurations of the build's baseline, in order.
WORKLOADS = {
    "c1_mha4_2k": Workload("c1_mha4_2k", 1, 4, 4, 2048, 2.0,
                           channel_profile="outlier4", perm_stat="absmax", seed=1000),
    "c2_llama7b_32k": Workload("c2_llama7b_32k", 1, 32, 32, 32768, 1.5, seed=1001),
    "c3_mistral7b_128k": Workload("c3_mistral7b_128k", 1, 32, 8, 131072, 1.5, seed=1002),
    "c4_llama7b_1m": Workload("c4_llama7b_1m", 1, 32, 32, 1048576, 1.5, seed=1003),
    "c5_batch16_32k": Workload("c5_batch16_32k", 16, 32, 32, 32768, 1.5, seed=1004),
}


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, stream]))


def channel_scales(w: Workload) -> tuple[np.ndarray, np.ndarray]:
    """Per-(kv head, channel) magnitude profile for K and for V, float32 [Hk][D]."""
    out = []
    for stream in (11, 12):
        r = _rng(w.seed, stream)
        if w.channel_profile == "loguniform":
            s = np.power(10.0, r.uniform(-1.0, 1.0, size=(w.n_kv_heads, w.head_dim)))
        elif w.channel_profile == "outlier4":
            s = np.ones((w.n_kv_heads, w.head_dim))
            for h in range(w.n_kv_heads):
                s[h, r.choice(w.head_dim, size=4, replace=False)] = 10.0
        else:
            raise ValueError(w.channel_profile)
        out.append(s.astype(np.float32))
    return out[0], out[1]


def make_kv(w: Workload, n_tokens: int | None = None, stream: int = 0) -> tuple[np.ndarray, np.ndarray]:
    """K and V as float16 [B][Hk][T][D] in the model's original channel order."""
    T = w.context if n_tokens is None else n_tokens
    sk, sv = channel_scales(w)
    res = []
    for i, s in enumerate((sk, sv)):
        r = _rng(w.seed, 100 + 2 * stream + i)
        x = np.empty((w.batch, w.n_kv_heads, T, w.head_dim), dtype=np.float16)
        for b in range(w.batch):
            for h in range(w.n_kv_heads):
                z = r.standard_normal(size=(T, w.head_dim), dtype=np.float32)
                x[b, h] = (z * s[h][None, :]).astype(np.float16)
        res.append(x)
    return res[0], res[1]


def make_kv_device(w: Workload, device, stream: int = 0):
    """The same distributions as make_kv, drawn on the GPU with a seeded torch.Generator (the
    host generator is too slow for the 1M-token and batch-16 workloads and for 32 layers).
    Returns K, V as torch float16 [B][Hk][T][D] on `device`, and the two reorder indices
    (int32 [Hk][D], channels sorted by their range over batch and sequence, ties by channel
    index) computed from them."""
    import torch

    sk, sv = channel_scales(w)
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed * 1000 + stream)
    shape = (w.batch, w.n_kv_heads, w.context, w.head_dim)
    out, perms = [], []
    for s in (sk, sv):
        s_d = torch.from_numpy(s).to(device)[None, :, None, :]
        x = torch.empty(shape, dtype=torch.float16, device=device)
        for b in range(w.batch):  # one sequence at a time bounds the fp32 temporaries
            z = torch.randn(shape[1:], generator=gen, device=device, dtype=torch.float32)
            x[b] = (z * s_d[0]).to(torch.float16)
            del z
        if w.perm_stat == "range":
            stat = x.amax(dim=(0, 2)).float() - x.amin(dim=(0, 2)).float()
        elif w.perm_stat == "absmax":
            stat = x.abs().amax(dim=(0, 2)).float()
        else:
            raise ValueError(w.perm_stat)
        perms.append(np.argsort(stat.cpu().numpy(), axis=-1, kind="stable").astype(np.int32))
        out.append(x)
    return out[0], out[1], perms[0], perms[1]


def make_query(w: Workload, stream: int = 0) -> np.ndarray:
    """One decode-step query, float16 [B][Hq][D]."""
    r = _rng(w.seed, 500 + stream)
    return r.standard_normal(size=(w.batch, w.n_q_heads, w.head_dim), dtype=np.float32).astype(np.float16)


def make_new_token(w: Workload, step: int) -> tuple[np.ndarray, np.ndarray]:
    """K and V of one newly generated token, float16 [B][Hk][D]."""
    sk, sv = channel_scales(w)
    res = []
    for i, s in enumerate((sk, sv)):
        r = _rng(w.seed, 10_000 + 2 * step + i)
        z = r.standard_normal(size=(w.batch, w.n_kv_heads, w.head_dim), dtype=np.float32)
        res.append((z * s[None]).astype(np.float16))
    return res[0], res[1]


def sort_permutation(x: np.ndarray, stat: str) -> np.ndarray:
    """Reorder index per kv head: channels in ascending order of a per-channel
    statistic taken over batch and sequence (ties broken by channel index).

    x: float16 [B][Hk][T][D]  ->  int32 [Hk][D], out[h][p] = source channel of
    permuted position p.
    """
    xf = x.astype(np.float32)
    if stat == "range":
        s = xf.max(axis=(0, 2)) - xf.min(axis=(0, 2))
    elif stat == "absmax":
        s = np.abs(xf).max(axis=(0, 2))
    else:
        raise ValueError(stat)
    return np.argsort(s, axis=-1, kind="stable").astype(np.int32)


def make_permutations(w: Workload, k: np.ndarray, v: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    return sort_permutation(k, w.perm_stat), sort_permutation(v, w.perm_stat)


def make_clip(w: Workload) -> tuple[np.ndarray, np.ndarray]:
    """Clip ratio per (kv head, group), float32 [Hk][D/G]; the paper calibrates
    it offline, the workloads use one constant."""
    shape = (w.n_kv_heads, w.head_dim // w.group_size)
    return np.full(shape, w.clip, np.float32), np.full(shape, w.clip, np.float32)
