"""ctypes front end of the LiteAttention CPU oracle -- TEST INFRASTRUCTURE.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import
this module; the product (the HIP library and its binding) never does, and this
module imports nothing of the product.

The arithmetic lives in ``lite_attn_oracle.c`` (Algorithm 2 of the paper with
the tile recurrences of its Preliminaries); this file only compiles it with gcc
and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lite_attn_oracle.c")
_LOCK = threading.Lock()
_LIBS: dict = {}


# LA_ORACLE_SANITIZE=1 (set by tests/test_sanitizers.py for a child process that preloads the sanitizer runtime):
# build and load an AddressSanitizer + UndefinedBehaviorSanitizer flavour of the same source instead
_SANITIZE = os.environ.get("LA_ORACLE_SANITIZE") == "1"


def _lib_path(f64: bool) -> str:
    return os.path.join(_HERE, "liblite_attn_oracle_%s%s.so" % ("f64" if f64 else "f32", "_san" if _SANITIZE else ""))


def build(force: bool = False) -> None:
    """Compile both precisions of the oracle with gcc (no fast-math: the sums keep their written order)."""
    for f64 in (False, True):
        out = _lib_path(f64)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra"]
        if _SANITIZE:
            cmd += ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g"]
        if f64:
            cmd.append("-DLA_ORACLE_F64")
        cmd += [_SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


class _Shape(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("seqlen", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("tile_q", ctypes.c_int32), ("tile_k", ctypes.c_int32),
        ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64),
        ("protect_start", ctypes.c_int32), ("protect_len", ctypes.c_int32), ("immediate", ctypes.c_int32),
    ]


def load_library(path: str, f64: bool):
    """dlopen a built oracle and declare its signatures (also used by the mutation tests, which build
    deliberately broken copies of the C source to show that the pins catch them)."""
    lib = ctypes.CDLL(path)
    real = ctypes.c_double if f64 else ctypes.c_float
    lib.la_oracle_step.restype = ctypes.c_int
    lib.la_oracle_step.argtypes = [
        ctypes.POINTER(_Shape), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_void_p, real, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    lib.la_oracle_real_bytes.restype = ctypes.c_int
    assert lib.la_oracle_real_bytes() == (8 if f64 else 4)
    return lib


def _load(f64: bool):
    with _LOCK:
        if f64 not in _LIBS:
            build()
            _LIBS[f64] = load_library(_lib_path(f64), f64)
        return _LIBS[f64]


def diagonal_first(tq: int, tk: int) -> np.ndarray:
    """Visiting order that starts at the diagonal tile and wraps around: i, i+1, ..., Tk-1, 0, ..., i-1."""
    return ((np.arange(tq)[:, None] + np.arange(tk)[None, :]) % tk).astype(np.int32)


def threads() -> int:
    """Number of OpenMP threads the oracle will use (for the benchmark's `cores` field)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        return int(env)
    return len(os.sched_getaffinity(0))


def oracle_step(q, k, v, mask, thr, *, tile_q=128, tile_k=128, protect=(0, 0), immediate=False,
                rows=None, f64=False, out=None, libs=None, visit=None):
    """One attention call of the oracle.

    q, k, v : uint16 numpy arrays [B,H,N,d] holding bf16 bit patterns (any strides with d contiguous).
    mask    : uint8 [B,H,Tq,Tk], nonzero = skipped on entry; NOT modified -- the exit mask is returned.
    thr     : signed threshold (-eps), natural-log units of S; ``-inf`` never fires.
    rows    : optional iterable of flattened row ids (b*H+h)*Tq+i; other rows of `out`/`g` stay NaN
              and their mask rows are returned unchanged.
    visit   : optional int32 [Tq,Tk], visit[i,t] = K/V tile that Q tile i visits t-th (default: ascending).
    Returns (out [B,H,N,d] real, mask_exit uint8, g [B,H,Tq,Tk] real with NaN for unevaluated tiles).
    """
    lib = libs[f64] if libs is not None else _load(f64)
    for a in (q, k, v):
        assert a.dtype == np.uint16 and a.ndim == 4 and a.strides[3] == 2
    assert q.shape == k.shape == v.shape and q.strides == k.strides == v.strides
    B, H, N, d = q.shape
    Tq, Tk = -(-N // tile_q), -(-N // tile_k)
    assert mask.shape == (B, H, Tq, Tk) and mask.dtype == np.uint8
    rdt = np.float64 if f64 else np.float32
    sh = _Shape(B, H, N, d, tile_q, tile_k, q.strides[0] // 2, q.strides[1] // 2, q.strides[2] // 2,
                int(protect[0]), int(protect[1]), 1 if immediate else 0)
    mask_exit = np.ascontiguousarray(mask).copy()
    if out is None:
        out = np.full((B, H, N, d), np.nan, dtype=rdt)
    g = np.full((B, H, Tq, Tk), np.nan, dtype=rdt)
    rows_arr = None
    if rows is not None:
        rows_arr = np.ascontiguousarray(np.asarray(list(rows), dtype=np.int64))
    visit_arr = None
    if visit is not None:
        visit_arr = np.ascontiguousarray(visit, dtype=np.int32)
        assert visit_arr.shape == (Tq, Tk) and (np.sort(visit_arr, axis=1) == np.arange(Tk)).all()
    rc = lib.la_oracle_step(ctypes.byref(sh), q.ctypes.data, k.ctypes.data, v.ctypes.data,
                            mask_exit.ctypes.data, float(thr), out.ctypes.data, g.ctypes.data,
                            rows_arr.ctypes.data if rows_arr is not None else None,
                            0 if rows_arr is None else rows_arr.size,
                            visit_arr.ctypes.data if visit_arr is not None else None)
    if rc != 0:
        raise ValueError("la_oracle_step failed with code %d" % rc)
    return out, mask_exit, g
