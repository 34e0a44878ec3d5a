"""ctypes front end of the CPU oracle (``adatopk_oracle.c``).

TEST INFRASTRUCTURE: only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this module.  It holds no arithmetic of
its own: every function marshals numpy arrays into the C routines, which state the
method as the paper's Sec. 5.1 (Top-K sparsification figure) and Sec. 5.2
(Eq. "adacompress") define it.  bf16 tensors travel as ``uint16`` bit patterns, fp16
tensors as ``float16`` arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adatopk_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_adatopk.so")

_lib = None


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc (host only).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle())
        i64, i32, p = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        lib.oracle_compress_f32.argtypes = [p, i64, i64, p, p, p]
        lib.oracle_compress_bf16.argtypes = [p, i64, i64, p, p, p]
        lib.oracle_compress_f16.argtypes = [p, i64, i64, p, p, p]
        lib.oracle_compress_segmented_f16.argtypes = [p, p, p, i32, p, p, p, p]
        lib.oracle_f16_to_f32.argtypes = [ctypes.c_uint16]
        lib.oracle_f16_to_f32.restype = ctypes.c_float
        for nm in ("f32", "bf16", "f16"):
            getattr(lib, "oracle_decompress_accumulate_" + nm).argtypes = [p, p, i64, p, i64]
        lib.oracle_round_bf16.argtypes = [ctypes.c_double]
        lib.oracle_round_bf16.restype = ctypes.c_uint16
        lib.oracle_round_f16.argtypes = [ctypes.c_double]
        lib.oracle_round_f16.restype = ctypes.c_uint16
        lib.oracle_decompress_f32.argtypes = [p, p, i64, p, i64]
        lib.oracle_decompress_bf16.argtypes = [p, p, i64, p, i64]
        lib.oracle_compress_segmented_f32.argtypes = [p, p, p, i32, p, p, p, p]
        lib.oracle_compress_segmented_bf16.argtypes = [p, p, p, i32, p, p, p, p]
        lib.oracle_adaptive_ratios.argtypes = [p, i32, ctypes.c_double, ctypes.c_double, p]
        lib.oracle_k_for_ratio.argtypes = [i64, ctypes.c_double]
        lib.oracle_k_for_ratio.restype = i64
        dbl = ctypes.c_double
        lib.oracle_link_time.argtypes = [dbl, dbl, dbl]
        lib.oracle_link_time.restype = dbl
        lib.oracle_pipeline_time.argtypes = [p, p, i32, i32]
        lib.oracle_pipeline_time.restype = dbl
        lib.oracle_pipeline_time_compressed.argtypes = [p, p, i32, i32, dbl, dbl, i32]
        lib.oracle_pipeline_time_compressed.restype = dbl
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _flat(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x).reshape(-1)
    if x.dtype not in (np.float32, np.uint16, np.float16):
        raise TypeError("oracle takes float32, float16, or uint16 holding bf16 bit patterns")
    return x


def _by_dtype(dt, f32, bf16, f16):
    return f32 if dt == np.float32 else (bf16 if dt == np.uint16 else f16)


def compress(x: np.ndarray, k: int):
    """(idx int32[k] ascending, val[k] same dtype as x, err float32) for one tensor."""
    x = _flat(x)
    k = int(k)
    idx = np.empty(k, dtype=np.int32)
    val = np.empty(k, dtype=x.dtype)
    err = np.zeros(1, dtype=np.float32)
    L = _load()
    fn = _by_dtype(x.dtype, L.oracle_compress_f32, L.oracle_compress_bf16, L.oracle_compress_f16)
    rc = fn(_ptr(x), x.size, k, _ptr(idx), _ptr(val), _ptr(err))
    if rc != 0:
        raise ValueError("oracle_compress: bad arguments (n=%d, k=%d)" % (x.size, k))
    return idx, val, np.float32(err[0])


def decompress(idx: np.ndarray, val: np.ndarray, n: int) -> np.ndarray:
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    val = _flat(val)
    y = np.empty(int(n), dtype=val.dtype)
    fn = _load().oracle_decompress_f32 if val.dtype == np.float32 else _load().oracle_decompress_bf16
    rc = fn(_ptr(idx), _ptr(val), idx.size, _ptr(y), int(n))
    if rc != 0:
        raise ValueError("oracle_decompress: index out of range or bad sizes")
    return y


def decompress_accumulate(idx: np.ndarray, val: np.ndarray, y: np.ndarray) -> np.ndarray:
    """Returns a copy of y with y[idx[j]] += val[j] (exact sum rounded once to the type)."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    val = _flat(val)
    out = _flat(y).copy()
    if out.dtype != val.dtype:
        raise TypeError("y and val must have one dtype")
    L = _load()
    fn = _by_dtype(val.dtype, L.oracle_decompress_accumulate_f32, L.oracle_decompress_accumulate_bf16,
                   L.oracle_decompress_accumulate_f16)
    if fn(_ptr(idx), _ptr(val), idx.size, _ptr(out), out.size) != 0:
        raise ValueError("oracle_decompress_accumulate: index out of range or bad sizes")
    return out


def round_bf16(s: float) -> int:
    return int(_load().oracle_round_bf16(float(s)))


def round_f16(s: float) -> int:
    return int(_load().oracle_round_f16(float(s)))


def compress_segmented(xs, ks):
    """Per-tensor compress of a list of tensors.  Returns (idx, val, out_offset, err[S])."""
    xs = [_flat(x) for x in xs]
    S = len(xs)
    dt = xs[0].dtype if S else np.float32
    ks = np.asarray(ks, dtype=np.int64).reshape(S)
    in_off = np.zeros(S + 1, dtype=np.int64)
    out_off = np.zeros(S + 1, dtype=np.int64)
    for s in range(S):
        in_off[s + 1] = in_off[s] + xs[s].size
        out_off[s + 1] = out_off[s] + ks[s]
    cat = np.concatenate(xs) if S else np.empty(0, dtype=dt)
    idx = np.empty(int(out_off[S]), dtype=np.int32)
    val = np.empty(int(out_off[S]), dtype=dt)
    err = np.zeros(max(S, 1), dtype=np.float32)
    L = _load()
    fn = _by_dtype(dt, L.oracle_compress_segmented_f32, L.oracle_compress_segmented_bf16,
                   L.oracle_compress_segmented_f16)
    rc = fn(_ptr(cat), _ptr(in_off), _ptr(ks), S, _ptr(idx), _ptr(val), _ptr(out_off), _ptr(err))
    if rc != 0:
        raise ValueError("oracle_compress_segmented: bad arguments")
    return idx, val, out_off, err[:S]


def f16_to_f32(bits: int) -> float:
    """IEEE binary16 pattern -> fp32 value, as the oracle widens it for the error norm."""
    return float(_load().oracle_f16_to_f32(int(bits) & 0xFFFF))


def adaptive_ratios(R, r: float, coeff: float = 3.0) -> np.ndarray:
    """Eq. "adacompress" (Sec. 5.2) for every link time in R."""
    R = np.ascontiguousarray(R, dtype=np.float64).reshape(-1)
    out = np.empty_like(R)
    rc = _load().oracle_adaptive_ratios(_ptr(R), R.size, float(r), float(coeff), _ptr(out))
    if rc != 0:
        raise ValueError("oracle_adaptive_ratios: bad arguments")
    return out


def k_for_ratio(n: int, r_i: float) -> int:
    return int(_load().oracle_k_for_ratio(int(n), float(r_i)))


def link_time(alpha: float, beta: float, nbytes: float) -> float:
    """Sec. 3.5: T_comm = alpha + beta * M."""
    return float(_load().oracle_link_time(float(alpha), float(beta), float(nbytes)))


def pipeline_time(C, R, n_b: int) -> float:
    """Sec. 3.6, Eq. "time_pipe"."""
    C = np.ascontiguousarray(C, dtype=np.float64)
    R = np.ascontiguousarray(R, dtype=np.float64)
    return float(_load().oracle_pipeline_time(_ptr(C), _ptr(R), C.size, int(n_b)))


def pipeline_time_compressed(C, R, n_b: int, r: float, coeff: float = 3.0, variant: int = 0) -> float:
    """Sec. 5.2, Eq. "time_pipe_compress"; variant 0 as printed, 1 with each link's own ratio in the last term."""
    C = np.ascontiguousarray(C, dtype=np.float64)
    R = np.ascontiguousarray(R, dtype=np.float64)
    return float(_load().oracle_pipeline_time_compressed(_ptr(C), _ptr(R), C.size, int(n_b), float(r), float(coeff),
                                                         int(variant)))
