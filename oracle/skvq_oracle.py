"""ctypes front end of the SKVQ CPU oracle: TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this.  It marshals numpy arrays into oracle/skvq_oracle.c and does no
arithmetic of its own.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libskvq_oracle.so")
_SRC = os.path.join(_HERE, "skvq_oracle.c")

HEAD_DIM = 128
VBLOCK = 32


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C11, one rounding per fp32 operation)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < max(
            os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "skvq_oracle.h"))):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


class _Config(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("group_size", C.c_int32), ("k_levels", C.c_int32),
                ("v_levels", C.c_int32), ("window", C.c_int32), ("n_sink", C.c_int32),
                ("meta_format", C.c_int32), ("max_quant_tokens", C.c_int64),
                ("perm_k", C.c_void_p), ("perm_v", C.c_void_p), ("clip_k", C.c_void_p),
                ("clip_v", C.c_void_p), ("sm_scale", C.c_float), ("group_bounds", C.c_void_p)]


class _Buffers(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("k_codes", "v_codes", "k_meta", "v_meta", "k_win", "v_win")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.skvq_ref_half_to_float.restype = C.c_float
        _lib.skvq_ref_half_to_float.argtypes = [C.c_uint16]
        _lib.skvq_ref_float_to_half.restype = C.c_uint16
        _lib.skvq_ref_float_to_half.argtypes = [C.c_float]
        _lib.skvq_ref_avg_bits.restype = C.c_double
        _lib.skvq_ref_avg_bits.argtypes = [C.c_double, C.c_int, C.c_int]
        _lib.skvq_ref_encode_group.restype = None
        _lib.skvq_ref_encode_group.argtypes = [C.c_void_p, C.c_int, C.c_float, C.c_int, C.c_int,
                                               C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.skvq_ref_float_to_e4m3.restype = C.c_uint8
        _lib.skvq_ref_float_to_e4m3.argtypes = [C.c_float]
        _lib.skvq_ref_e4m3_to_float.restype = C.c_float
        _lib.skvq_ref_e4m3_to_float.argtypes = [C.c_uint8]
        _lib.skvq_ref_round_meta.restype = C.c_float
        _lib.skvq_ref_round_meta.argtypes = [C.c_float, C.c_int]
        _lib.skvq_ref_k_get.argtypes = [C.c_void_p, C.c_int, C.c_int]
        _lib.skvq_ref_k_put.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int]
        _lib.skvq_ref_k_put.restype = None
        _lib.skvq_ref_v_get.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int]
        _lib.skvq_ref_v_put.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int]
        _lib.skvq_ref_v_put.restype = None
        _lib.skvq_ref_sizes.restype = None
        _lib.skvq_ref_sizes.argtypes = [C.c_void_p, C.c_void_p]
        _lib.skvq_ref_prefill_quantize.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                   C.c_int64, C.c_void_p]
        _lib.skvq_ref_quantize_append.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                  C.c_void_p]
        _lib.skvq_ref_decode_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                                   C.c_void_p, C.c_void_p]
        _lib.skvq_ref_prefill_quantize_filtered.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                            C.c_int64, C.c_void_p, C.c_void_p]
        _lib.skvq_ref_quantize_append_filtered.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                           C.c_void_p, C.c_void_p]
        _lib.skvq_ref_decode_attention_filtered.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                                            C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        _lib.skvq_ref_calibrate_clip.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                                 C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                                 C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.skvq_ref_decode_attention_multi.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int,
                                                         C.c_void_p, C.c_void_p]
        _lib.skvq_ref_channel_stats.restype = None
        _lib.skvq_ref_channel_stats.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int64, C.c_void_p]
        _lib.skvq_ref_calibrate_reorder.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                                    C.c_void_p]
        _lib.skvq_ref_prefill_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                                    C.c_void_p]
        _lib.skvq_ref_prefill_attention_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                                         C.c_void_p, C.c_int64, C.c_void_p]
    return _lib


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def half_to_float(bits: int) -> float:
    return float(lib().skvq_ref_half_to_float(int(bits)))


def float_to_half(x: float) -> int:
    return int(lib().skvq_ref_float_to_half(float(x)))


def avg_bits(code_bits: float, meta_bits: int, group_size: int) -> float:
    return float(lib().skvq_ref_avg_bits(code_bits, meta_bits, group_size))


META_FORMATS = {"f32": 0, "f16": 1, "e4m3": 2}
META_DTYPES = {0: np.float32, 1: np.float16, 2: np.uint8}


def float_to_e4m3(x: float) -> int:
    return int(lib().skvq_ref_float_to_e4m3(float(x)))


def e4m3_to_float(b: int) -> float:
    return float(lib().skvq_ref_e4m3_to_float(int(b)))


def round_meta(x: float, meta: str) -> float:
    return float(lib().skvq_ref_round_meta(float(x), META_FORMATS[meta]))


def encode_group(xp: np.ndarray, alpha: float, levels: int, meta: str = "f32"):
    """Eq. 2 on one group of already reordered float32 values."""
    xp = np.ascontiguousarray(xp, dtype=np.float32)
    codes = np.zeros(xp.size, np.uint8)
    scale = np.zeros(1, np.float32)
    zero = np.zeros(1, np.float32)
    lib().skvq_ref_encode_group(_ptr(xp), xp.size, float(alpha), int(levels), META_FORMATS[meta],
                                _ptr(codes), _ptr(scale), _ptr(zero))
    return codes, scale[0], zero[0]


def channel_stats(x: np.ndarray) -> np.ndarray:
    """(min, max) per (kv head, channel) of fp16 x [B][Hk][T][D] -> float32 [Hk][D][2]."""
    x = np.ascontiguousarray(x)
    assert x.dtype == np.float16 and x.ndim == 4 and x.shape[3] == HEAD_DIM
    stats = np.zeros((x.shape[1], HEAD_DIM, 2), np.float32)
    lib().skvq_ref_channel_stats(_ptr(x), x.shape[0], x.shape[1], x.shape[2], _ptr(stats))
    return stats


def calibrate_reorder(stats: np.ndarray, group_size: int, granularity: int = 1, max_iter: int = 100):
    """KMeans reorder: returns (perm [Hk][D], bounds [Hk][D/G + 1])."""
    stats = np.ascontiguousarray(stats, np.float32)
    hk = stats.shape[0]
    perm = np.zeros((hk, HEAD_DIM), np.int32)
    bounds = np.zeros((hk, HEAD_DIM // group_size + 1), np.int32)
    rc = lib().skvq_ref_calibrate_reorder(_ptr(stats), hk, group_size, granularity, max_iter, _ptr(perm), _ptr(bounds))
    if rc != 0:
        raise RuntimeError(f"oracle reorder calibration failed: {rc}")
    return perm, bounds


def levels_of(bits: float) -> int:
    return {4.0: 16, 3.0: 8, 2.0: 4, 1.5: 3}[float(bits)]


class OracleCache:
    """Host-side mixed-precision cache of one attention layer, driven by the oracle."""

    def __init__(self, batch, n_q_heads, n_kv_heads, group_size, v_bits, window, max_quant_tokens,
                 perm_k, perm_v, clip_k, clip_v, sm_scale=None, k_bits=2.0, fill=0, n_sink=0,
                 meta="f32", group_bounds=None):
        self.perm_k = np.ascontiguousarray(perm_k, np.int32)
        self.perm_v = np.ascontiguousarray(perm_v, np.int32)
        self.clip_k = np.ascontiguousarray(clip_k, np.float32)
        self.clip_v = np.ascontiguousarray(clip_v, np.float32)
        if sm_scale is None:
            sm_scale = 1.0 / np.sqrt(HEAD_DIM)
        # unequal groups: per kv head HEAD_DIM // group_size + 1 ascending boundaries (group_size = the
        # average); one row is repeated for every kv head
        self.group_bounds = None
        if group_bounds is not None:
            gb = np.atleast_2d(np.asarray(group_bounds, np.int32))
            if gb.shape[0] == 1:
                gb = np.repeat(gb, n_kv_heads, axis=0)
            self.group_bounds = np.ascontiguousarray(gb)
            assert self.group_bounds.shape == (n_kv_heads, HEAD_DIM // group_size + 1)
        self.cfg = _Config(batch, n_q_heads, n_kv_heads, HEAD_DIM, group_size, levels_of(k_bits),
                           levels_of(v_bits), window, n_sink, META_FORMATS[meta], max_quant_tokens,
                           _ptr(self.perm_k),
                           _ptr(self.perm_v), _ptr(self.clip_k), _ptr(self.clip_v), sm_scale,
                           None if self.group_bounds is None else _ptr(self.group_bounds))
        sizes = (C.c_size_t * 6)()
        lib().skvq_ref_sizes(C.byref(self.cfg), sizes)
        self.sizes = [int(s) for s in sizes]
        ng = HEAD_DIM // group_size
        heads = batch * n_kv_heads
        nblk = (max_quant_tokens + VBLOCK - 1) // VBLOCK
        vb = {3: 832, 4: 1024, 8: 1536, 16: 2048}[levels_of(v_bits)]
        kb = {4: 32, 8: 48, 16: 64}[levels_of(k_bits)]
        self.k_codes = np.full((batch, n_kv_heads, max_quant_tokens, kb), fill, np.uint8)
        self.v_codes = np.full((batch, n_kv_heads, nblk, vb), fill, np.uint8)
        mdt = META_DTYPES[META_FORMATS[meta]]   # fp8 values are kept as their bytes
        self.meta = meta
        self.k_meta = np.zeros((batch, n_kv_heads, max_quant_tokens, ng, 2), mdt)
        self.v_meta = np.zeros((batch, n_kv_heads, max_quant_tokens, ng, 2), mdt)
        self.k_win = np.zeros((batch, n_kv_heads, window + n_sink, HEAD_DIM), np.uint16)
        self.v_win = np.zeros((batch, n_kv_heads, window + n_sink, HEAD_DIM), np.uint16)
        for a in (self.k_meta, self.v_meta, self.k_win, self.v_win):
            a.view(np.uint8)[...] = fill     # untouched bytes keep the caller's initial pattern
        assert [a.nbytes for a in self.arrays()] == self.sizes, (self.sizes, heads)
        self.buf = _Buffers(*[_ptr(a) for a in self.arrays()])
        self.n_tokens = 0
        self.keep = None     # filter mask over the tokens that have left the window (None: the sink rule a < S)
        self.window = window
        self.n_sink = n_sink
        self.shape = (batch, n_q_heads, n_kv_heads)

    def arrays(self):
        return [self.k_codes, self.v_codes, self.k_meta, self.v_meta, self.k_win, self.v_win]

    @property
    def n_quant(self) -> int:
        left = max(self.n_tokens - self.window, 0)
        if self.keep is not None:
            return left - int(np.count_nonzero(self.keep[:left]))
        return max(left - self.n_sink, 0)

    def _keep_array(self, n: int) -> np.ndarray:
        """The mask as a contiguous uint8 array of at least n (and at least one) entries."""
        a = np.zeros(max(n, 1), np.uint8)
        a[:len(self.keep)] = self.keep[:len(a)]
        return a

    def prefill(self, k: np.ndarray, v: np.ndarray, keep=None) -> int:
        """keep (optional): one entry per token older than the window, nonzero = kept in fp16 (a filter rule's
        decision); without it the first n_sink tokens are kept."""
        if keep is not None:
            b, _, hk = self.shape
            T = k.shape[2]
            keep = np.asarray(keep).astype(bool).astype(np.uint8)
            assert keep.shape == (max(T - self.window, 0),)
            k, v = np.ascontiguousarray(k), np.ascontiguousarray(v)
            old = self.keep
            self.keep = keep.copy()
            n = C.c_int64(0)
            km = self._keep_array(len(keep))   # (kept alive across the call)
            rc = lib().skvq_ref_prefill_quantize_filtered(C.byref(self.cfg), C.byref(self.buf), _ptr(k), _ptr(v), T,
                                                          _ptr(km), C.byref(n))
            if rc == 0:
                self.n_tokens = n.value
            else:
                self.keep = old
            return rc
        self.keep = None
        b, _, hk = self.shape
        assert k.dtype == np.float16 and v.dtype == np.float16
        assert k.shape == v.shape and k.shape[:2] == (b, hk) and k.shape[3] == HEAD_DIM
        k = np.ascontiguousarray(k)
        v = np.ascontiguousarray(v)
        n = C.c_int64(0)
        rc = lib().skvq_ref_prefill_quantize(C.byref(self.cfg), C.byref(self.buf), _ptr(k), _ptr(v),
                                             k.shape[2], C.byref(n))
        if rc == 0:
            self.n_tokens = n.value
        return rc

    def append(self, k_new: np.ndarray, v_new: np.ndarray, keep=None) -> int:
        """keep (optional): the filter rules' decision for the token that leaves the window in this step."""
        b, _, hk = self.shape
        assert k_new.dtype == np.float16 and k_new.shape == (b, hk, HEAD_DIM) == v_new.shape
        k_new = np.ascontiguousarray(k_new)
        v_new = np.ascontiguousarray(v_new)
        n = C.c_int64(self.n_tokens)
        if keep is not None or self.keep is not None:
            left = max(self.n_tokens - self.window, 0)
            mask = self.keep if self.keep is not None else (np.arange(left) < self.n_sink).astype(np.uint8)
            leaving = self.n_tokens >= self.window
            if leaving:
                # without a decision: the sink rule (keep token a if a < S and a row is free)
                decision = bool(keep) if keep is not None else (left < self.n_sink and int(np.count_nonzero(mask[:left])) < self.n_sink)
                mask = np.concatenate([mask[:left], np.array([decision], np.uint8)])
            old, self.keep = self.keep, mask
            km = self._keep_array(len(mask))
            rc = lib().skvq_ref_quantize_append_filtered(C.byref(self.cfg), C.byref(self.buf), _ptr(k_new),
                                                         _ptr(v_new), _ptr(km), C.byref(n))
            if rc == 0:
                self.n_tokens = n.value
            else:
                self.keep = old
            return rc
        rc = lib().skvq_ref_quantize_append(C.byref(self.cfg), C.byref(self.buf), _ptr(k_new),
                                            _ptr(v_new), C.byref(n))
        if rc == 0:
            self.n_tokens = n.value
        return rc

    def decode(self, q: np.ndarray, want_f16: bool = False):
        b, hq, _ = self.shape
        assert q.dtype == np.float16 and q.shape == (b, hq, HEAD_DIM)
        q = np.ascontiguousarray(q)
        out = np.zeros((b, hq, HEAD_DIM), np.float32)
        out16 = np.zeros((b, hq, HEAD_DIM), np.float16) if want_f16 else None
        if self.keep is not None:
            km = self._keep_array(len(self.keep))
            rc = lib().skvq_ref_decode_attention_filtered(C.byref(self.cfg), C.byref(self.buf), self.n_tokens,
                                                          _ptr(km), _ptr(q), 1, _ptr(out),
                                                          _ptr(out16) if want_f16 else None)
        else:
            rc = lib().skvq_ref_decode_attention(C.byref(self.cfg), C.byref(self.buf), self.n_tokens,
                                                 _ptr(q), _ptr(out), _ptr(out16) if want_f16 else None)
        if rc != 0:
            raise RuntimeError(f"oracle decode failed: {rc}")
        return (out, out16) if want_f16 else out

    def decode_multi(self, q: np.ndarray) -> np.ndarray:
        """q [B][n_new][Hq][D]: query token j sees the cached tokens 0 .. T - n_new + j."""
        b, hq, _ = self.shape
        assert q.dtype == np.float16 and q.ndim == 4 and q.shape[0] == b and q.shape[2:] == (hq, HEAD_DIM)
        q = np.ascontiguousarray(q)
        out = np.zeros(q.shape, np.float32)
        if self.keep is not None:
            km = self._keep_array(len(self.keep))
            rc = lib().skvq_ref_decode_attention_filtered(C.byref(self.cfg), C.byref(self.buf), self.n_tokens,
                                                          _ptr(km), _ptr(q), q.shape[1], _ptr(out), None)
        else:
            rc = lib().skvq_ref_decode_attention_multi(C.byref(self.cfg), C.byref(self.buf), self.n_tokens, _ptr(q),
                                                       q.shape[1], _ptr(out), None)
        if rc != 0:
            raise RuntimeError(f"oracle multi-token decode failed: {rc}")
        return out

    def prefill_attention(self, q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
        """Causal attention of the prompt on the fp16 inputs; q [B][Hq][T][D], k/v [B][Hk][T][D]."""
        b, hq, hk = self.shape
        T = q.shape[2]
        assert q.dtype == k.dtype == v.dtype == np.float16
        assert q.shape == (b, hq, T, HEAD_DIM) and k.shape == v.shape == (b, hk, T, HEAD_DIM)
        q, k, v = (np.ascontiguousarray(x) for x in (q, k, v))
        out = np.zeros((b, hq, T, HEAD_DIM), np.float32)
        rc = lib().skvq_ref_prefill_attention(C.byref(self.cfg), _ptr(q), _ptr(k), _ptr(v), T, _ptr(out))
        if rc != 0:
            raise RuntimeError(f"oracle prefill attention failed: {rc}")
        return out

    def prefill_attention_rows(self, q: np.ndarray, k: np.ndarray, v: np.ndarray, rows) -> np.ndarray:
        """Chosen rows of the prompt's causal attention: rows is a list of (sequence, query head, query);
        returns [len(rows)][D]."""
        b, hq, hk = self.shape
        T = q.shape[2]
        assert q.dtype == k.dtype == v.dtype == np.float16
        assert q.shape == (b, hq, T, HEAD_DIM) and k.shape == v.shape == (b, hk, T, HEAD_DIM)
        q, k, v = (np.ascontiguousarray(x) for x in (q, k, v))
        rows = np.ascontiguousarray(np.asarray(rows, np.int64).reshape(-1, 3))
        out = np.zeros((rows.shape[0], HEAD_DIM), np.float32)
        rc = lib().skvq_ref_prefill_attention_rows(C.byref(self.cfg), _ptr(q), _ptr(k), _ptr(v), T, _ptr(rows),
                                                   rows.shape[0], _ptr(out))
        if rc != 0:
            raise RuntimeError(f"oracle prefill attention (rows) failed: {rc}")
        return out

    def calibrate_clip(self, k, v, q, o_ref, alphas):
        """Eq. 3 by one pass of coordinate descent over `alphas`; returns (clip_k, clip_v, loss[Hk]).
        k, v [B][Hk][T][D] fp16; q [n][B][Hq][D] fp16; o_ref [n][B][Hq][D] f32."""
        b, hq, hk = self.shape
        ng = self.clip_k.shape[1]
        k, v, q = (np.ascontiguousarray(x) for x in (k, v, q))
        o_ref = np.ascontiguousarray(o_ref, np.float32)
        alphas = np.ascontiguousarray(alphas, np.float32)
        assert q.shape[1:] == (b, hq, HEAD_DIM) and o_ref.shape == q.shape and k.shape == v.shape
        ck, cv = np.zeros((hk, ng), np.float32), np.zeros((hk, ng), np.float32)
        loss = np.zeros(hk, np.float64)
        rc = lib().skvq_ref_calibrate_clip(C.byref(self.cfg), C.byref(self.buf), _ptr(k), _ptr(v), k.shape[2],
                                           _ptr(q), q.shape[0], _ptr(o_ref), _ptr(alphas), alphas.size,
                                           _ptr(ck), _ptr(cv), _ptr(loss))
        if rc != 0:
            raise RuntimeError(f"oracle clip calibration failed: {rc}")
        return ck, cv, loss

    # format accessors, for tests that look inside the packed buffers
    def k_code(self, b, h, t, p) -> int:
        row = self.k_codes[b, h, t]
        return int(lib().skvq_ref_k_get(_ptr(row), self.cfg.k_levels, p))

    def v_code(self, b, h, t, p) -> int:
        blk = self.v_codes[b, h, t // VBLOCK]
        return int(lib().skvq_ref_v_get(_ptr(blk), self.cfg.v_levels, t % VBLOCK, p))


def num_threads() -> int:
    return int(lib().skvq_ref_num_threads())
