"""Run under LD_PRELOAD=libasan: drives the sanitizer build of the library's host side (fake device on the host heap,
see hip/hip_runtime.h here) through a whole handle / context life cycle, so that every host-side copy, allocation and
release runs under AddressSanitizer and UndefinedBehaviorSanitizer.  Usage: lifecycle.py <library.so>"""
import ctypes
import sys

import numpy as np

lib = ctypes.CDLL(sys.argv[1])
H = ctypes.c_void_p


class Desc(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("seqlen", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("tile_q", ctypes.c_int32), ("tile_k", ctypes.c_int32),
                ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64),
                ("protect_start", ctypes.c_int32), ("protect_len", ctypes.c_int32),
                ("flags", ctypes.c_int32), ("max_steps", ctypes.c_int32)]


class Stats(ctypes.Structure):
    _fields_ = [("step", ctypes.c_int32), ("tiles_total", ctypes.c_uint64), ("tiles_skipped_in", ctypes.c_uint64),
                ("tiles_newly_marked", ctypes.c_uint64), ("live_list_bytes", ctypes.c_uint64)]


lib.lite_attn_mask_words.restype = ctypes.c_size_t
lib.lite_attn_mask_words.argtypes = [H]
lib.lite_attn_skipruns_stride.restype = ctypes.c_size_t
lib.lite_attn_skipruns_stride.argtypes = [H]
lib.lite_attn_free_mask.restype = None
lib.lite_attn_free_mask.argtypes = [H]
lib.lite_attn_fwd.argtypes = [ctypes.c_void_p] * 4 + [H, ctypes.c_float, ctypes.c_int]
lib.lite_attn_mask_export.argtypes = [H, ctypes.c_void_p, ctypes.c_size_t]
lib.lite_attn_mask_import.argtypes = [H, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
lib.lite_attn_skipruns_export.argtypes = [H, ctypes.c_void_p, ctypes.c_void_p]
lib.lite_attn_skiplist_export.argtypes = [H, ctypes.c_void_p, ctypes.c_void_p]
lib.lite_attn_skip_stats.argtypes = [H, ctypes.c_int, ctypes.POINTER(Stats)]
lib.lite_attn_kernel_times.argtypes = [H, ctypes.c_int, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float)]
lib.lite_attn_profile.argtypes = [H, ctypes.c_int]
lib.lite_attn_set_stream.argtypes = [H, ctypes.c_void_p]
lib.lite_attn_init_mask.argtypes = [ctypes.POINTER(Desc), ctypes.POINTER(H)]
lib.lite_attn_init_mask_shared.argtypes = [ctypes.POINTER(Desc), H, ctypes.POINTER(H)]
lib.lite_attn_ctx_create.argtypes = [ctypes.POINTER(H)]
lib.lite_attn_ctx_set_stream.argtypes = [H, ctypes.c_void_p]
lib.lite_attn_ctx_free.argtypes = [H]


def desc(heads, n, steps=3, flags=0, protect=(0, 0)):
    return Desc(1, heads, n, 128, 128, 128, heads * n * 128, n * 128, 128, protect[0], protect[1], flags, steps)


def exercise(h, heads, n, steps):
    tk = -(-n // 128)
    rows = heads * tk
    words = lib.lite_attn_mask_words(h)
    assert words == rows * (-(-tk // 64))
    buf = (ctypes.c_uint8 * (heads * n * 128 * 2 + 16))()
    p = (ctypes.addressof(buf) + 15) & ~15
    assert lib.lite_attn_fwd(p, p, p, p + 1, h, ctypes.c_float(-1.0), 0) == -1          # misaligned
    assert lib.lite_attn_fwd(p, p, p, p, h, ctypes.c_float(0.0), 0) == -1               # threshold >= 0
    assert lib.lite_attn_fwd(p, p, p, p, h, ctypes.c_float(float("nan")), 0) == -1
    assert lib.lite_attn_fwd(p, p, p, p, h, ctypes.c_float(-1.0), 2) == -2              # step out of sequence
    assert lib.lite_attn_profile(h, 1) == 0
    for t in range(steps):
        assert lib.lite_attn_fwd(p, p, p, p, h, ctypes.c_float(-1.0), t) == 0
    assert lib.lite_attn_fwd(p, p, p, p, h, ctypes.c_float(-1.0), steps) == -2          # >= max_steps
    st = Stats()
    assert lib.lite_attn_skip_stats(h, steps - 1, ctypes.byref(st)) == 0 and st.tiles_total == rows * tk
    assert lib.lite_attn_skip_stats(h, steps, ctypes.byref(st)) == -2
    a, b = ctypes.c_float(), ctypes.c_float()
    assert lib.lite_attn_kernel_times(h, 0, ctypes.byref(a), ctypes.byref(b)) == 0
    bits = np.zeros(words, dtype=np.uint64)
    assert lib.lite_attn_mask_export(h, bits.ctypes.data, words) == 0
    assert lib.lite_attn_mask_export(h, bits.ctypes.data, words + 1) == -1
    bits[:] = 5
    assert lib.lite_attn_mask_import(h, bits.ctypes.data, words, 1) == 0
    assert lib.lite_attn_mask_import(h, bits.ctypes.data, words, steps) == -2
    back = np.zeros(words, dtype=np.uint64)
    assert lib.lite_attn_mask_export(h, back.ctypes.data, words) == 0 and (back == 5).all()
    stride = lib.lite_attn_skipruns_stride(h)
    assert stride == tk // 2 + 1
    runs = np.zeros((rows, stride), dtype=np.uint32)
    nruns = np.zeros(rows, dtype=np.uint32)
    assert lib.lite_attn_skipruns_export(h, runs.ctypes.data, nruns.ctypes.data) == 0 and (nruns == 1).all()
    idx = np.zeros((rows, tk), dtype=np.uint16)
    cnt = np.zeros(rows, dtype=np.uint32)
    assert lib.lite_attn_skiplist_export(h, idx.ctypes.data, cnt.ctypes.data) == 0
    assert (cnt == tk).all() and (idx == np.arange(tk, dtype=np.uint16)).all()


for heads, n in ((1, 1), (2, 300), (3, 128 * 65 + 7)):
    for flags in (0, 1, 2, 3):
        h = H()
        d = desc(heads, n, flags=flags, protect=(0, min(n, 5)))
        assert lib.lite_attn_init_mask(ctypes.byref(d), ctypes.byref(h)) == 0
        assert lib.lite_attn_set_stream(h, None) == 0
        exercise(h, heads, n, 3)
        lib.lite_attn_free_mask(h)

ctx = H()
assert lib.lite_attn_ctx_create(ctypes.byref(ctx)) == 0
assert lib.lite_attn_ctx_set_stream(ctx, ctypes.c_void_p(64)) == 0
hs = []
for heads, n in ((2, 300), (1, 128 * 9), (4, 2000), (1, 50)):       # the shared scratch grows twice
    h = H()
    d = desc(heads, n)
    assert lib.lite_attn_init_mask_shared(ctypes.byref(d), ctx, ctypes.byref(h)) == 0
    hs.append((h, heads, n))
assert lib.lite_attn_init_mask_shared(ctypes.byref(desc(1, 10)), None, ctypes.byref(H())) == -1
assert lib.lite_attn_set_stream(hs[0][0], ctypes.c_void_p(64)) == 0
assert lib.lite_attn_set_stream(hs[0][0], ctypes.c_void_p(128)) == -6
assert lib.lite_attn_ctx_free(ctx) == -6
for h, heads, n in hs:
    exercise(h, heads, n, 3)
for h, _, _ in hs:
    lib.lite_attn_free_mask(h)
assert lib.lite_attn_ctx_free(ctx) == 0
assert lib.lite_attn_ctx_free(None) == 0
print("lifecycle ok")
