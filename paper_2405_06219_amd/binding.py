"""Thin ctypes binding of libskvq.so (include/skvq.h): argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch is used to own device
memory and to name the current stream.  There is no fallback: if the library has not been
built, importing a function from here raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libskvq.so")

SKVQ_OK = 0
SKVQ_ERR_INVALID_ARG, SKVQ_ERR_UNSUPPORTED, SKVQ_ERR_CAPACITY, SKVQ_ERR_STATE, SKVQ_ERR_HIP = -1, -2, -3, -4, -5
SKVQ_BITS_4, SKVQ_BITS_3, SKVQ_BITS_2, SKVQ_BITS_1P5 = 16, 8, 4, 3
SKVQ_MAX_SPLITS = 128
SKVQ_STATIC_MAX_ROWS = 64
HEAD_DIM = 128
BUFFER_NAMES = ("k_codes", "v_codes", "k_meta", "v_meta", "k_win", "v_win", "workspace")


class skvq_config(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("group_size", C.c_int32), ("k_bits", C.c_int32),
                ("v_bits", C.c_int32), ("window", C.c_int32), ("n_sink", C.c_int32),
                ("meta_format", C.c_int32), ("max_quant_tokens", C.c_int64),
                ("perm_k", C.c_void_p), ("perm_v", C.c_void_p), ("clip_k", C.c_void_p),
                ("clip_v", C.c_void_p), ("sm_scale", C.c_float), ("max_new_tokens", C.c_int32),
                ("group_bounds", C.c_void_p)]


class skvq_buffers(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in BUFFER_NAMES]


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2405_06219_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.skvq_sizes.argtypes = [C.POINTER(skvq_config), C.POINTER(C.c_size_t)]
        L.skvq_validate_config.argtypes = [C.POINTER(skvq_config)]
        L.skvq_create.argtypes = [C.POINTER(skvq_config), C.POINTER(skvq_buffers), C.POINTER(C.c_void_p)]
        L.skvq_destroy.argtypes = [C.c_void_p]
        L.skvq_destroy.restype = None
        L.skvq_prefill_quantize.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.skvq_calibrate_channel_stats.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p]
        L.skvq_calibrate_reorder.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                             C.c_void_p]
        L.skvq_decode_attention_multi.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.skvq_set_clip.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.skvq_calibrate_clip.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32,
                                          C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_void_p]
        L.skvq_prefill_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                             C.c_void_p, C.c_void_p, C.c_void_p]
        L.skvq_prefill_attention_quantize.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                                      C.c_void_p, C.c_void_p, C.c_void_p]
        L.skvq_quantize_append.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.skvq_prefill_quantize_filtered.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                                     C.c_void_p]
        L.skvq_quantize_append_filtered.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        L.skvq_decode_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.skvq_decode_attention_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.skvq_append_decode_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                   C.c_void_p, C.c_void_p]
        L.skvq_get_state.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int32)]
        L.skvq_set_state.argtypes = [C.c_void_p, C.c_int64]
        L.skvq_set_num_splits.argtypes = [C.c_void_p, C.c_int32]
        L.skvq_read_yardstick.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.skvq_read_write_yardstick.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p]
        L.skvq_status_string.argtypes = [C.c_int]
        L.skvq_status_string.restype = C.c_char_p
        L.skvq_last_error.argtypes = [C.c_void_p]
        L.skvq_last_error.restype = C.c_char_p
        _lib = L
    return _lib


class SkvqError(RuntimeError):
    def __init__(self, status: int, detail: str = ""):
        self.status = status
        text = lib().skvq_status_string(status).decode()
        super().__init__(f"skvq status {status} ({text}) {detail}".strip())


META_FORMATS = {"f32": 0, "f16": 1, "e4m3": 2}   # skvq_meta_format
META_DTYPES = {0: np.float32, 1: np.float16, 2: np.uint8}


def bits_enum(bits: float) -> int:
    return {4.0: SKVQ_BITS_4, 3.0: SKVQ_BITS_3, 2.0: SKVQ_BITS_2, 1.5: SKVQ_BITS_1P5}[float(bits)]


def make_config(batch, n_q_heads, n_kv_heads, group_size, v_bits, window, max_quant_tokens, perm_k, perm_v,
                clip_k, clip_v, sm_scale=0.0, k_bits=2.0, head_dim=HEAD_DIM, n_sink=0, meta="f32",
                group_bounds=None, max_new_tokens=0):
    """Returns (skvq_config, keepalive): the numpy arrays the config points to."""
    keep = [np.ascontiguousarray(perm_k, np.int32), np.ascontiguousarray(perm_v, np.int32),
            np.ascontiguousarray(clip_k, np.float32), np.ascontiguousarray(clip_v, np.float32)]
    if group_bounds is not None:      # [n_kv_heads][head_dim / group_size + 1]; one row serves every head
        gb = np.atleast_2d(np.asarray(group_bounds, np.int32))
        if gb.shape[0] == 1:
            gb = np.repeat(gb, n_kv_heads, axis=0)
        keep.append(np.ascontiguousarray(gb))
        if keep[4].shape != (n_kv_heads, head_dim // group_size + 1):
            raise ValueError("group_bounds needs head_dim / group_size + 1 entries per kv head")
    cfg = skvq_config(batch, n_q_heads, n_kv_heads, head_dim, group_size, bits_enum(k_bits), bits_enum(v_bits),
                      window, n_sink, META_FORMATS[meta], max_quant_tokens, keep[0].ctypes.data, keep[1].ctypes.data, keep[2].ctypes.data,
                      keep[3].ctypes.data, float(sm_scale), int(max_new_tokens),
                      keep[4].ctypes.data if group_bounds is not None else None)
    return cfg, keep


def skvq_sizes(cfg: skvq_config) -> list[int]:
    out = (C.c_size_t * 7)()
    rc = lib().skvq_sizes(C.byref(cfg), out)
    if rc != SKVQ_OK:
        raise SkvqError(rc)
    return [int(x) for x in out]


def skvq_calibrate_channel_stats(x: torch.Tensor, stream=None) -> np.ndarray:
    """(min, max) per (kv head, channel) of fp16 x [B][Hk][T][D] on the device -> float32 [Hk][D][2]."""
    b, hk, T, d = x.shape
    xp = _dev_ptr(x, torch.float16, (b, hk, T, HEAD_DIM))
    stats = np.zeros((hk, HEAD_DIM, 2), np.float32)
    rc = lib().skvq_calibrate_channel_stats(xp, b, hk, T, stats.ctypes.data, _stream_ptr(stream))
    if rc != SKVQ_OK:
        raise SkvqError(rc)
    return stats


def skvq_calibrate_reorder(stats: np.ndarray, group_size: int, granularity: int = 16, max_iter: int = 100):
    """KMeans channel reorder: returns (perm [Hk][D], bounds [Hk][D/G + 1])."""
    stats = np.ascontiguousarray(stats, np.float32)
    hk = stats.shape[0]
    perm = np.zeros((hk, HEAD_DIM), np.int32)
    bounds = np.zeros((hk, HEAD_DIM // group_size + 1), np.int32)
    rc = lib().skvq_calibrate_reorder(stats.ctypes.data, hk, group_size, granularity, max_iter, perm.ctypes.data,
                                      bounds.ctypes.data)
    if rc != SKVQ_OK:
        raise SkvqError(rc)
    return perm, bounds


def skvq_read_yardstick(src: torch.Tensor, sink: torch.Tensor, stream=None):
    """The library's read-only kernel over the bytes of `src` (a contiguous device tensor)."""
    rc = lib().skvq_read_yardstick(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _stream_ptr(stream))
    if rc != SKVQ_OK:
        raise SkvqError(rc)


def skvq_read_write_yardstick(src: torch.Tensor, dst: torch.Tensor, ratio: int, stream=None):
    """The library's read/write kernel: reads ratio times the bytes of `dst` from `src` and fills `dst`
    (contiguous device tensors; `src` must hold at least that many bytes)."""
    nbytes = dst.numel() * dst.element_size()
    if src.numel() * src.element_size() < ratio * nbytes:
        raise SkvqError(SKVQ_ERR_INVALID_ARG)
    rc = lib().skvq_read_write_yardstick(src.data_ptr(), dst.data_ptr(), nbytes, ratio, _stream_ptr(stream))
    if rc != SKVQ_OK:
        raise SkvqError(rc)


def skvq_validate_config(cfg: skvq_config) -> int:
    return int(lib().skvq_validate_config(C.byref(cfg)))


def _stream_ptr(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dev_ptr(t: torch.Tensor, dtype, shape) -> int:
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype and tuple(t.shape) == tuple(shape)):
        raise ValueError(f"expected contiguous cuda {dtype} tensor of shape {tuple(shape)}, got {t.dtype} "
                         f"{tuple(t.shape)} on {t.device}")
    return t.data_ptr()


class SkvqCache:
    """One layer's cache: owns the device buffers (torch tensors) and the library handle."""

    def __init__(self, batch, n_q_heads, n_kv_heads, group_size, v_bits, window, max_quant_tokens, perm_k, perm_v,
                 clip_k, clip_v, sm_scale=0.0, k_bits=2.0, device="cuda:0", fill=None, n_sink=0,
                 meta="f32", group_bounds=None, max_new_tokens=0):
        self.cfg, self._keep = make_config(batch, n_q_heads, n_kv_heads, group_size, v_bits, window,
                                           max_quant_tokens, perm_k, perm_v, clip_k, clip_v, sm_scale, k_bits,
                                           n_sink=n_sink, meta=meta, group_bounds=group_bounds,
                                           max_new_tokens=max_new_tokens)
        self.shape = (batch, n_q_heads, n_kv_heads)
        self.window = window
        self.device = torch.device(device)
        self.sizes = skvq_sizes(self.cfg)
        self.buffers = {}
        for name, nbytes in zip(BUFFER_NAMES, self.sizes):
            t = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            if fill is not None:
                t.fill_(fill)
            self.buffers[name] = t
        self._bufs = skvq_buffers(*[self.buffers[n].data_ptr() for n in BUFFER_NAMES])
        handle = C.c_void_p()
        with torch.cuda.device(self.device):
            rc = lib().skvq_create(C.byref(self.cfg), C.byref(self._bufs), C.byref(handle))
        if rc != SKVQ_OK:
            raise SkvqError(rc)
        self._h = handle

    def close(self):
        if getattr(self, "_h", None):
            lib().skvq_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != SKVQ_OK:
            raise SkvqError(rc, lib().skvq_last_error(self._h).decode())

    # ---- clip scales: Eq. 2's alpha, and its calibration by Eq. 3 ----
    def skvq_set_clip(self, clip_k: np.ndarray, clip_v: np.ndarray, stream=None):
        ck = np.ascontiguousarray(clip_k, np.float32)
        cv = np.ascontiguousarray(clip_v, np.float32)
        ng = HEAD_DIM // self.cfg.group_size
        if ck.shape != (self.shape[2], ng) or cv.shape != ck.shape:
            raise ValueError("clip scales must be [n_kv_heads][head_dim / group_size]")
        self._check(lib().skvq_set_clip(self._h, ck.ctypes.data, cv.ctypes.data, _stream_ptr(stream)))

    def skvq_calibrate_clip(self, k: torch.Tensor, v: torch.Tensor, q: torch.Tensor, o_ref: torch.Tensor,
                            alphas, stream=None):
        """Returns (clip_k, clip_v, loss) as numpy arrays [Hk][NG], [Hk][NG], [Hk]."""
        b, hq, hk = self.shape
        T, n = k.shape[2], q.shape[0]
        kp = _dev_ptr(k, torch.float16, (b, hk, T, HEAD_DIM))
        vp = _dev_ptr(v, torch.float16, (b, hk, T, HEAD_DIM))
        qp = _dev_ptr(q, torch.float16, (n, b, hq, HEAD_DIM))
        op = _dev_ptr(o_ref, torch.float32, (n, b, hq, HEAD_DIM))
        al = np.ascontiguousarray(alphas, np.float32)
        ng = HEAD_DIM // self.cfg.group_size
        ck, cv = np.zeros((hk, ng), np.float32), np.zeros((hk, ng), np.float32)
        loss = np.zeros(hk, np.float64)
        self._check(lib().skvq_calibrate_clip(self._h, kp, vp, T, qp, n, op, al.ctypes.data, al.size, ck.ctypes.data,
                                              cv.ctypes.data, loss.ctypes.data, _stream_ptr(stream)))
        return ck, cv, loss

    # ---- the hot-path calls, named as in the C ABI ----
    def skvq_prefill_attention(self, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                               out_f32: torch.Tensor | None = None, out_f16: torch.Tensor | None = None,
                               stream=None) -> torch.Tensor:
        b, hq, hk = self.shape
        T = q.shape[2]
        qp = _dev_ptr(q, torch.float16, (b, hq, T, HEAD_DIM))
        kp = _dev_ptr(k, torch.float16, (b, hk, T, HEAD_DIM))
        vp = _dev_ptr(v, torch.float16, (b, hk, T, HEAD_DIM))
        if out_f32 is None:
            out_f32 = torch.empty((b, hq, T, HEAD_DIM), dtype=torch.float32, device=self.device)
        op = _dev_ptr(out_f32, torch.float32, (b, hq, T, HEAD_DIM))
        o16 = _dev_ptr(out_f16, torch.float16, (b, hq, T, HEAD_DIM)) if out_f16 is not None else None
        self._check(lib().skvq_prefill_attention(self._h, qp, kp, vp, T, op, o16, _stream_ptr(stream)))
        return out_f32

    def skvq_prefill_attention_quantize(self, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                                        out_f32: torch.Tensor | None = None, out_f16: torch.Tensor | None = None,
                                        stream=None) -> torch.Tensor:
        b, hq, hk = self.shape
        T = q.shape[2]
        qp = _dev_ptr(q, torch.float16, (b, hq, T, HEAD_DIM))
        kp = _dev_ptr(k, torch.float16, (b, hk, T, HEAD_DIM))
        vp = _dev_ptr(v, torch.float16, (b, hk, T, HEAD_DIM))
        if out_f32 is None:
            out_f32 = torch.empty((b, hq, T, HEAD_DIM), dtype=torch.float32, device=self.device)
        op = _dev_ptr(out_f32, torch.float32, (b, hq, T, HEAD_DIM))
        o16 = _dev_ptr(out_f16, torch.float16, (b, hq, T, HEAD_DIM)) if out_f16 is not None else None
        self._check(lib().skvq_prefill_attention_quantize(self._h, qp, kp, vp, T, op, o16, _stream_ptr(stream)))
        return out_f32

    def skvq_prefill_quantize(self, k: torch.Tensor, v: torch.Tensor, stream=None):
        b, _, hk = self.shape
        T = k.shape[2]
        kp = _dev_ptr(k, torch.float16, (b, hk, T, HEAD_DIM))
        vp = _dev_ptr(v, torch.float16, (b, hk, T, HEAD_DIM))
        self._check(lib().skvq_prefill_quantize(self._h, kp, vp, T, _stream_ptr(stream)))

    def skvq_prefill_quantize_filtered(self, k: torch.Tensor, v: torch.Tensor, keep, stream=None):
        """keep: one entry per token older than the window (host array-like; nonzero = kept in fp16) or None."""
        b, _, hk = self.shape
        T = k.shape[2]
        kp = _dev_ptr(k, torch.float16, (b, hk, T, HEAD_DIM))
        vp = _dev_ptr(v, torch.float16, (b, hk, T, HEAD_DIM))
        mask = None
        if keep is not None:
            mask = np.ascontiguousarray(np.asarray(keep).astype(bool).astype(np.uint8))
            if mask.shape != (max(T - self.window, 0),):
                raise ValueError("keep must have one entry per token older than the window")
            if mask.size == 0:
                mask = np.zeros(1, np.uint8)
        self._check(lib().skvq_prefill_quantize_filtered(self._h, kp, vp, T, mask.ctypes.data if mask is not None else None,
                                                         _stream_ptr(stream)))

    def skvq_quantize_append_filtered(self, k_new: torch.Tensor, v_new: torch.Tensor, keep_leaving: bool, stream=None):
        b, _, hk = self.shape
        kp = _dev_ptr(k_new, torch.float16, (b, hk, HEAD_DIM))
        vp = _dev_ptr(v_new, torch.float16, (b, hk, HEAD_DIM))
        self._check(lib().skvq_quantize_append_filtered(self._h, kp, vp, 1 if keep_leaving else 0, _stream_ptr(stream)))

    def skvq_quantize_append(self, k_new: torch.Tensor, v_new: torch.Tensor, stream=None):
        b, _, hk = self.shape
        kp = _dev_ptr(k_new, torch.float16, (b, hk, HEAD_DIM))
        vp = _dev_ptr(v_new, torch.float16, (b, hk, HEAD_DIM))
        self._check(lib().skvq_quantize_append(self._h, kp, vp, _stream_ptr(stream)))

    def skvq_decode_attention(self, q: torch.Tensor, out_f32: torch.Tensor | None = None,
                              out_f16: torch.Tensor | None = None, stream=None) -> torch.Tensor:
        b, hq, _ = self.shape
        qp = _dev_ptr(q, torch.float16, (b, hq, HEAD_DIM))
        if out_f32 is None:
            out_f32 = torch.empty((b, hq, HEAD_DIM), dtype=torch.float32, device=self.device)
        op = _dev_ptr(out_f32, torch.float32, (b, hq, HEAD_DIM))
        hp = _dev_ptr(out_f16, torch.float16, (b, hq, HEAD_DIM)) if out_f16 is not None else None
        self._check(lib().skvq_decode_attention(self._h, qp, op, hp, _stream_ptr(stream)))
        return out_f32

    def skvq_decode_attention_static(self, q: torch.Tensor, out_f32: torch.Tensor, out_f16: torch.Tensor | None = None,
                                     stream=None) -> torch.Tensor:
        """The variant that allocates nothing: the caller passes the output tensor too."""
        b, hq, _ = self.shape
        qp = _dev_ptr(q, torch.float16, (b, hq, HEAD_DIM))
        op = _dev_ptr(out_f32, torch.float32, (b, hq, HEAD_DIM))
        hp = _dev_ptr(out_f16, torch.float16, (b, hq, HEAD_DIM)) if out_f16 is not None else None
        self._check(lib().skvq_decode_attention_static(self._h, qp, op, hp, _stream_ptr(stream)))
        return out_f32

    def skvq_append_decode_attention(self, k_new: torch.Tensor, v_new: torch.Tensor, q: torch.Tensor,
                                     out_f32: torch.Tensor | None = None, out_f16: torch.Tensor | None = None,
                                     stream=None) -> torch.Tensor:
        b, hq, hk = self.shape
        kp = _dev_ptr(k_new, torch.float16, (b, hk, HEAD_DIM))
        vp = _dev_ptr(v_new, torch.float16, (b, hk, HEAD_DIM))
        qp = _dev_ptr(q, torch.float16, (b, hq, HEAD_DIM))
        if out_f32 is None:
            out_f32 = torch.empty((b, hq, HEAD_DIM), dtype=torch.float32, device=self.device)
        op = _dev_ptr(out_f32, torch.float32, (b, hq, HEAD_DIM))
        hp = _dev_ptr(out_f16, torch.float16, (b, hq, HEAD_DIM)) if out_f16 is not None else None
        self._check(lib().skvq_append_decode_attention(self._h, kp, vp, qp, op, hp, _stream_ptr(stream)))
        return out_f32

    # ---- state ----
    def skvq_get_state(self):
        a, b, c = C.c_int64(), C.c_int64(), C.c_int32()
        self._check(lib().skvq_get_state(self._h, C.byref(a), C.byref(b), C.byref(c)))
        return a.value, b.value, c.value

    def skvq_set_state(self, n_tokens: int):
        self._check(lib().skvq_set_state(self._h, n_tokens))

    def skvq_set_num_splits(self, n: int):
        self._check(lib().skvq_set_num_splits(self._h, n))

    def skvq_decode_attention_multi(self, q: torch.Tensor, out_f32: torch.Tensor | None = None,
                                    out_f16: torch.Tensor | None = None, stream=None) -> torch.Tensor:
        """q [B][n_new][Hq][D]: the last n_new cached tokens' queries; returns fp32 [B][n_new][Hq][D]."""
        b, hq, _ = self.shape
        n_new = q.shape[1]
        qp = _dev_ptr(q, torch.float16, (b, n_new, hq, HEAD_DIM))
        if out_f32 is None:
            out_f32 = torch.empty((b, n_new, hq, HEAD_DIM), dtype=torch.float32, device=self.device)
        op = _dev_ptr(out_f32, torch.float32, (b, n_new, hq, HEAD_DIM))
        o16 = _dev_ptr(out_f16, torch.float16, (b, n_new, hq, HEAD_DIM)) if out_f16 is not None else None
        self._check(lib().skvq_decode_attention_multi(self._h, qp, n_new, op, o16, _stream_ptr(stream)))
        return out_f32

    # ---- views of the buffers for tests ----
    def host_arrays(self):
        """Buffers copied to the host with the shapes the format statement gives them."""
        b, _, hk = self.shape
        tcap = self.cfg.max_quant_tokens
        ng = HEAD_DIM // self.cfg.group_size
        vb = {SKVQ_BITS_1P5: 832, SKVQ_BITS_2: 1024, SKVQ_BITS_3: 1536, SKVQ_BITS_4: 2048}[self.cfg.v_bits]
        kb = {SKVQ_BITS_2: 32, SKVQ_BITS_3: 48, SKVQ_BITS_4: 64}[self.cfg.k_bits]
        torch.cuda.synchronize(self.device)
        raw = {n: self.buffers[n].cpu().numpy() for n in BUFFER_NAMES[:6]}
        return [raw["k_codes"].reshape(b, hk, tcap, kb),
                raw["v_codes"].reshape(b, hk, (tcap + 31) // 32, vb),
                raw["k_meta"].view(META_DTYPES[self.cfg.meta_format]).reshape(b, hk, tcap, ng, 2),
                raw["v_meta"].view(META_DTYPES[self.cfg.meta_format]).reshape(b, hk, tcap, ng, 2),
                raw["k_win"].view(np.uint16).reshape(b, hk, self.cfg.window + self.cfg.n_sink, HEAD_DIM),
                raw["v_win"].view(np.uint16).reshape(b, hk, self.cfg.window + self.cfg.n_sink, HEAD_DIM)]
