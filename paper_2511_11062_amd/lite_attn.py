"""Thin ctypes binding of the C ABI in include/lite_attn.h (same names, argument marshalling only).

Every step of the attention path runs in the HIP library; there is no fallback: importing this module
without the built ``liblite_attn.so`` raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblite_attn.so")

if not os.path.exists(LIB_PATH):
    raise ImportError("liblite_attn.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
_lib = ctypes.CDLL(LIB_PATH)


class Desc(ctypes.Structure):
    """lite_attn_desc_t"""
    _fields_ = [
        ("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("seqlen", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("tile_q", ctypes.c_int32), ("tile_k", ctypes.c_int32),
        ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64),
        ("protect_start", ctypes.c_int32), ("protect_len", ctypes.c_int32),
        ("flags", ctypes.c_int32), ("max_steps", ctypes.c_int32),
    ]


class Stats(ctypes.Structure):
    """lite_attn_stats_t"""
    _fields_ = [
        ("step", ctypes.c_int32), ("tiles_total", ctypes.c_uint64), ("tiles_skipped_in", ctypes.c_uint64),
        ("tiles_newly_marked", ctypes.c_uint64), ("live_list_bytes", ctypes.c_uint64),
    ]


# desc.flags (include/lite_attn.h)
LITE_ATTN_PV_SKIP_IMMEDIATE = 1
LITE_ATTN_ORDER_DIAGONAL_FIRST = 2

_H = ctypes.c_void_p
_lib.lite_attn_init_mask.argtypes = [ctypes.POINTER(Desc), ctypes.POINTER(_H)]
_lib.lite_attn_set_stream.argtypes = [_H, ctypes.c_void_p]
_lib.lite_attn_fwd.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, _H,
                               ctypes.c_float, ctypes.c_int]
_lib.lite_attn_skip_stats.argtypes = [_H, ctypes.c_int, ctypes.POINTER(Stats)]
_lib.lite_attn_mask_words.argtypes = [_H]
_lib.lite_attn_mask_words.restype = ctypes.c_size_t
_lib.lite_attn_mask_export.argtypes = [_H, ctypes.c_void_p, ctypes.c_size_t]
_lib.lite_attn_mask_import.argtypes = [_H, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
_lib.lite_attn_skiplist_export.argtypes = [_H, ctypes.c_void_p, ctypes.c_void_p]
_lib.lite_attn_skipruns_export.argtypes = [_H, ctypes.c_void_p, ctypes.c_void_p]
_lib.lite_attn_skipruns_export.restype = ctypes.c_int
_lib.lite_attn_skipruns_stride.argtypes = [_H]
_lib.lite_attn_skipruns_stride.restype = ctypes.c_size_t
_lib.lite_attn_profile.argtypes = [_H, ctypes.c_int]
_lib.lite_attn_kernel_times.argtypes = [_H, ctypes.c_int, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float)]
_lib.lite_attn_fwd_static.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.POINTER(Desc), ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p]
_lib.lite_attn_fwd_static.restype = ctypes.c_int
_lib.lite_attn_ctx_create.argtypes = [ctypes.POINTER(_H)]
_lib.lite_attn_ctx_set_stream.argtypes = [_H, ctypes.c_void_p]
_lib.lite_attn_init_mask_shared.argtypes = [ctypes.POINTER(Desc), _H, ctypes.POINTER(_H)]
_lib.lite_attn_ctx_free.argtypes = [_H]
_lib.lite_attn_free_mask.argtypes = [_H]
_lib.lite_attn_free_mask.restype = None
_lib.lite_attn_strerror.argtypes = [ctypes.c_int]
_lib.lite_attn_strerror.restype = ctypes.c_char_p
_lib.lite_attn_last_hip_error.restype = ctypes.c_int
for _n in ("init_mask", "set_stream", "fwd", "skip_stats", "mask_export", "mask_import", "skiplist_export",
           "profile", "kernel_times", "ctx_create", "ctx_set_stream", "init_mask_shared", "ctx_free"):
    getattr(_lib, "lite_attn_" + _n).restype = ctypes.c_int


class LiteAttnError(RuntimeError):
    def __init__(self, code):
        self.code = code
        msg = _lib.lite_attn_strerror(code).decode()
        if code == -5:
            msg += " (hipError_t %d)" % _lib.lite_attn_last_hip_error()
        super().__init__("lite_attn: %s [%d]" % (msg, code))


def _check(rc):
    if rc != 0:
        raise LiteAttnError(rc)


def make_desc(batch, heads, seqlen, *, head_dim=128, tile_q=128, tile_k=128, strides=None, protect=(0, 0),
              max_steps=64, flags=0) -> Desc:
    """lite_attn_desc_t.  `strides` = (stride_b, stride_h, stride_n) in elements; default [B,H,N,d] contiguous."""
    if strides is None:
        strides = (heads * seqlen * head_dim, seqlen * head_dim, head_dim)
    return Desc(batch, heads, seqlen, head_dim, tile_q, tile_k, strides[0], strides[1], strides[2],
                int(protect[0]), int(protect[1]), flags, max_steps)


def lite_attn_init_mask(batch, heads, seqlen, **desc_fields):
    """-> opaque handle (keyword arguments: see make_desc)."""
    desc = make_desc(batch, heads, seqlen, **desc_fields)
    h = _H()
    _check(_lib.lite_attn_init_mask(ctypes.byref(desc), ctypes.byref(h)))
    return h


def lite_attn_ctx_create():
    """-> opaque context whose handles share one per-call scratch and one stream."""
    c = _H()
    _check(_lib.lite_attn_ctx_create(ctypes.byref(c)))
    return c


def lite_attn_ctx_set_stream(ctx, hip_stream):
    _check(_lib.lite_attn_ctx_set_stream(ctx, ctypes.c_void_p(int(hip_stream))))


def lite_attn_init_mask_shared(ctx, batch, heads, seqlen, **desc_fields):
    """-> opaque handle attached to `ctx` (keyword arguments: see make_desc)."""
    desc = make_desc(batch, heads, seqlen, **desc_fields)
    h = _H()
    _check(_lib.lite_attn_init_mask_shared(ctypes.byref(desc), ctx, ctypes.byref(h)))
    return h


def lite_attn_ctx_free(ctx):
    _check(_lib.lite_attn_ctx_free(ctx))


def lite_attn_set_stream(mask, hip_stream):
    """`hip_stream`: integer value of a hipStream_t (e.g. torch.cuda.current_stream().cuda_stream)."""
    _check(_lib.lite_attn_set_stream(mask, ctypes.c_void_p(int(hip_stream))))


def lite_attn_fwd(q, k, v, out, skip_mask, threshold, step):
    """q, k, v, out: integer device addresses (e.g. tensor.data_ptr()) of bf16 buffers."""
    _check(_lib.lite_attn_fwd(ctypes.c_void_p(int(q)), ctypes.c_void_p(int(k)), ctypes.c_void_p(int(v)),
                              ctypes.c_void_p(int(out)), skip_mask, ctypes.c_float(threshold), int(step)))


def lite_attn_fwd_static(q, k, v, out, desc: Desc, dev_skip_mask, threshold, hip_stream):
    """The allocation-free call.  q, k, v, out, dev_skip_mask: integer device addresses; `desc` from make_desc;
    dev_skip_mask holds static_mask_words(desc) uint64 words owned by the caller."""
    _check(_lib.lite_attn_fwd_static(ctypes.c_void_p(int(q)), ctypes.c_void_p(int(k)), ctypes.c_void_p(int(v)),
                                     ctypes.c_void_p(int(out)), ctypes.byref(desc), ctypes.c_void_p(int(dev_skip_mask)),
                                     ctypes.c_float(threshold), ctypes.c_void_p(int(hip_stream))))


def static_mask_words(desc: Desc) -> int:
    """uint64 words of the Skip-Mask of a layer: B*H*Tq*ceil(Tk/64)."""
    tq, tk = -(-desc.seqlen // desc.tile_q), -(-desc.seqlen // desc.tile_k)
    return desc.batch * desc.heads * tq * (-(-tk // 64))


def lite_attn_skip_stats(mask, step) -> Stats:
    st = Stats()
    _check(_lib.lite_attn_skip_stats(mask, int(step), ctypes.byref(st)))
    return st


def lite_attn_mask_words(mask) -> int:
    return int(_lib.lite_attn_mask_words(mask))


def lite_attn_mask_export(mask) -> np.ndarray:
    """-> uint64 numpy array of lite_attn_mask_words() words ([B*H*Tq][ceil(Tk/64)] flattened)."""
    bits = np.empty(lite_attn_mask_words(mask), dtype=np.uint64)
    _check(_lib.lite_attn_mask_export(mask, bits.ctypes.data, bits.size))
    return bits


def lite_attn_mask_import(mask, bits: np.ndarray, next_step: int):
    bits = np.ascontiguousarray(bits, dtype=np.uint64)
    _check(_lib.lite_attn_mask_import(mask, bits.ctypes.data, bits.size, int(next_step)))


def lite_attn_skiplist_export(mask, rows: int, tk: int):
    """-> (live_idx uint16 [rows,tk], live_cnt uint32 [rows]) of the current mask."""
    idx = np.empty((rows, tk), dtype=np.uint16)
    cnt = np.empty(rows, dtype=np.uint32)
    _check(_lib.lite_attn_skiplist_export(mask, idx.ctypes.data, cnt.ctypes.data))
    return idx, cnt


def lite_attn_profile(mask, enable: bool):
    _check(_lib.lite_attn_profile(mask, 1 if enable else 0))


def lite_attn_kernel_times(mask, step):
    """-> (prep_ms, attention_ms) of a completed step that ran with profiling enabled; prep = Skip-List compaction
    + V transposition pre-pass."""
    a, b = ctypes.c_float(), ctypes.c_float()
    _check(_lib.lite_attn_kernel_times(mask, int(step), ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def lite_attn_skipruns_export(mask, rows: int):
    """-> (runs uint32 [rows, stride] with start | end << 16 per run, nruns uint32 [rows]) of the current mask."""
    stride = int(_lib.lite_attn_skipruns_stride(mask))
    runs = np.empty((rows, stride), dtype=np.uint32)
    nruns = np.empty(rows, dtype=np.uint32)
    _check(_lib.lite_attn_skipruns_export(mask, runs.ctypes.data, nruns.ctypes.data))
    return runs, nruns


def lite_attn_skipruns_stride(mask) -> int:
    """Entries per row of the run-length Skip-List."""
    return int(_lib.lite_attn_skipruns_stride(mask))


def lite_attn_free_mask(mask):
    _lib.lite_attn_free_mask(mask)


def lite_attn_strerror(code: int) -> str:
    return _lib.lite_attn_strerror(int(code)).decode()
