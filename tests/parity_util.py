"""Builds the same cache twice -- CPU oracle and HIP library -- from one set of seeded inputs."""
from __future__ import annotations

import numpy as np
import torch

from oracle import skvq_oracle as O
from paper_2405_06219_amd import binding as B
from paper_2405_06219_amd import synth

TOL = 2e-3  # max-abs bound on attention outputs (fp32), the build's stated floating-point bar


def log(msg: str):
    """Progress line on stdout, flushed (names the case that was running if a run ends without a report)."""
    print(msg, flush=True)


class Pair:
    def __init__(self, w: synth.Workload, max_quant_tokens: int, perm_k, perm_v, clip_k, clip_v, sm_scale=0.0,
                 fill=0xAB, device="cuda:0", n_sink=0, meta="f32", group_bounds=None, max_new_tokens=0):
        self.w = w
        osm = sm_scale if sm_scale else None
        self.ref = O.OracleCache(w.batch, w.n_q_heads, w.n_kv_heads, w.group_size, w.v_bits, w.window,
                                 max_quant_tokens, perm_k, perm_v, clip_k, clip_v, sm_scale=osm, fill=fill,
                                 n_sink=n_sink, meta=meta, k_bits=w.k_bits, group_bounds=group_bounds)
        self.gpu = B.SkvqCache(w.batch, w.n_q_heads, w.n_kv_heads, w.group_size, w.v_bits, w.window,
                               max_quant_tokens, perm_k, perm_v, clip_k, clip_v, sm_scale=sm_scale, fill=fill,
                               device=device, n_sink=n_sink, meta=meta, k_bits=w.k_bits,
                               group_bounds=group_bounds, max_new_tokens=max_new_tokens)
        self.device = device

    def prefill(self, k: np.ndarray, v: np.ndarray):
        assert self.ref.prefill(k, v) == 0
        self.gpu.skvq_prefill_quantize(torch.from_numpy(k).to(self.device), torch.from_numpy(v).to(self.device))
        torch.cuda.synchronize()

    def append(self, k_new: np.ndarray, v_new: np.ndarray):
        assert self.ref.append(k_new, v_new) == 0
        self.gpu.skvq_quantize_append(torch.from_numpy(k_new).to(self.device), torch.from_numpy(v_new).to(self.device))

    def prefill_filtered(self, k: np.ndarray, v: np.ndarray, keep):
        assert self.ref.prefill(k, v, keep=keep) == 0
        self.gpu.skvq_prefill_quantize_filtered(torch.from_numpy(k).to(self.device), torch.from_numpy(v).to(self.device), keep)
        torch.cuda.synchronize()

    def append_filtered(self, k_new: np.ndarray, v_new: np.ndarray, keep: bool):
        assert self.ref.append(k_new, v_new, keep=keep) == 0
        self.gpu.skvq_quantize_append_filtered(torch.from_numpy(k_new).to(self.device),
                                               torch.from_numpy(v_new).to(self.device), keep)

    def assert_buffers_equal(self):
        names = ["k_codes", "v_codes", "k_meta", "v_meta", "k_win", "v_win"]
        got = self.gpu.host_arrays()
        assert self.gpu.skvq_get_state()[0] == self.ref.n_tokens
        for name, g, r in zip(names, got, self.ref.arrays()):
            if g.dtype == np.float32:       # compare bit patterns (distinguishes -0 from +0)
                g, r = g.view(np.uint32), r.view(np.uint32)
            elif g.dtype == np.float16:
                g, r = g.view(np.uint16), r.view(np.uint16)
            if not np.array_equal(g, r):
                bad = np.argwhere(g != r)
                raise AssertionError(f"{name}: {len(bad)} mismatches, first at {bad[0].tolist()}: "
                                     f"gpu {g[tuple(bad[0])]} oracle {r[tuple(bad[0])]}")

    def decode_both(self, q: np.ndarray, want_f16=False):
        ref = self.ref.decode(q, want_f16=want_f16)
        qd = torch.from_numpy(q).to(self.device)
        o16 = torch.empty(q.shape, dtype=torch.float16, device=self.device) if want_f16 else None
        out = self.gpu.skvq_decode_attention(qd, out_f16=o16)
        torch.cuda.synchronize()
        if want_f16:
            return (out.cpu().numpy(), o16.cpu().numpy()), ref
        return out.cpu().numpy(), ref


    def append_decode_both(self, k_new: np.ndarray, v_new: np.ndarray, q: np.ndarray):
        """One decode step as a single library call against the oracle's append followed by its decode."""
        assert self.ref.append(k_new, v_new) == 0
        ref = self.ref.decode(q)
        out = self.gpu.skvq_append_decode_attention(torch.from_numpy(k_new).to(self.device),
                                                    torch.from_numpy(v_new).to(self.device),
                                                    torch.from_numpy(q).to(self.device))
        torch.cuda.synchronize()
        return out.cpu().numpy(), ref


def make_pair(w: synth.Workload, extra_tokens: int = 0, **kw):
    """Pair + its seeded inputs (k, v, q) for workload w."""
    k, v = synth.make_kv(w)
    ks, vs = (k, v) if w.context else synth.make_kv(w, n_tokens=64)   # statistics for the permutation
    pk, pv = synth.make_permutations(w, ks, vs)
    ck, cv = synth.make_clip(w)
    tcap = max(w.context - w.window + extra_tokens, 1)
    pair = Pair(w, tcap, pk, pv, ck, cv, **kw)
    return pair, k, v, synth.make_query(w)
