"""Python names for the C ABI of ``libadatopk.so`` (see ``include/adatopk.h``).

Argument marshalling only: every step of compress / decompress runs in the HIP kernels of
the library.  torch supplies device memory and the current stream.  There is no fallback:
if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# ADATOPK_LIBRARY selects another build of the same C ABI (for instance one compiled with
# different launch-shape constants); the default is the in-tree library.
LIB_PATH = os.environ.get("ADATOPK_LIBRARY") or os.path.join(_HERE, "libadatopk.so")

F32, BF16, F16 = 0, 1, 2
OK, EINVAL, EWORKSPACE, ERUNTIME, ENOTIMPL = 0, 1, 2, 3, 4
_STATUS = {OK: "ADATOPK_OK", EINVAL: "ADATOPK_EINVAL", EWORKSPACE: "ADATOPK_EWORKSPACE",
           ERUNTIME: "ADATOPK_ERUNTIME", ENOTIMPL: "ADATOPK_ENOTIMPL"}

MEASURE_LIB_PATH = os.environ.get("ADATOPK_MEASURE_LIBRARY") or os.path.join(_HERE, "libadatopk_measure.so")

_lib = None          # the product library
_measure_lib = None  # the same sources built with the benchmark's timing hooks (adatopk_measure.h)
_active = None       # what load_library() returns when set: the measuring build inside `with measuring()`


class AdaTopKError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__("%s returned %s" % (where, _STATUS.get(status, status)))
        self.status = status


def load_library() -> ctypes.CDLL:
    global _lib
    if _active is not None:
        return _active
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libadatopk.so is not built: run `python -m paper_2410_12707_amd.build` "
                          "(or __graft_entry__.build()) first; there is no CPU fallback")
    _lib = _declare(ctypes.CDLL(LIB_PATH))
    return _lib


def load_measure_library() -> ctypes.CDLL:
    """The measuring build: the whole C ABI plus the hooks of adatopk_measure.h (benchmarks only)."""
    global _measure_lib
    if _measure_lib is not None:
        return _measure_lib
    if not os.path.exists(MEASURE_LIB_PATH):
        raise ImportError("libadatopk_measure.so is not built: run `python -m paper_2410_12707_amd.build`")
    lib = _declare(ctypes.CDLL(MEASURE_LIB_PATH))
    i32, p, sz = ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t
    lib.adatopk_measure_enable.argtypes = [i32]
    lib.adatopk_measure_enable.restype = i32
    lib.adatopk_measure_stage_count.restype = i32
    lib.adatopk_measure_stage_name.argtypes = [i32]
    lib.adatopk_measure_stage_name.restype = ctypes.c_char_p
    lib.adatopk_measure_read.argtypes = [p]
    lib.adatopk_measure_read.restype = i32
    lib.adatopk_measure_copy.argtypes = [p, p, sz, p]
    lib.adatopk_measure_copy.restype = i32
    lib.adatopk_measure_read_only.argtypes = [p, sz, p, p]
    lib.adatopk_measure_read_only.restype = i32
    lib.adatopk_measure_fill.argtypes = [p, sz, p]
    lib.adatopk_measure_fill.restype = i32
    _measure_lib = lib
    return lib


class measuring:
    """``with measuring():`` routes every call of this module through the measuring build and times each
    kernel launch with events of its own; ``measure_read()`` inside the block returns the durations."""

    def __enter__(self):
        global _active
        lib = load_measure_library()
        _check(lib.adatopk_measure_enable(1), "adatopk_measure_enable")
        _active = lib
        return self

    def __exit__(self, *exc):
        global _active
        _active = None
        _check(load_measure_library().adatopk_measure_enable(0), "adatopk_measure_enable")
        return False


def _declare(lib: ctypes.CDLL) -> ctypes.CDLL:
    i64, i32, p, sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t
    lib.adatopk_workspace_bytes.argtypes = [i64, i32, i32]
    lib.adatopk_workspace_bytes.restype = sz
    lib.adatopk_compress.argtypes = [p, i64, i32, i64, p, p, p, p, sz, p]
    lib.adatopk_compress.restype = i32
    lib.adatopk_decompress.argtypes = [p, p, i64, i32, p, i64, p]
    lib.adatopk_decompress.restype = i32
    lib.adatopk_decompress_sorted.argtypes = [p, p, i64, i32, p, i64, p]
    lib.adatopk_decompress_sorted.restype = i32
    lib.adatopk_decompress_accumulate.argtypes = [p, p, i64, i32, p, i64, p]
    lib.adatopk_decompress_accumulate.restype = i32
    lib.adatopk_decompress_segmented.argtypes = [p, p, p, i32, i32, p, p, p]
    lib.adatopk_decompress_segmented.restype = i32
    lib.adatopk_wire_bytes.argtypes = [i64, i32, i32]
    lib.adatopk_wire_bytes.restype = sz
    lib.adatopk_wire_keep_count.argtypes = [sz, i32, i32]
    lib.adatopk_wire_keep_count.restype = i64
    lib.adatopk_wire_parse_header.argtypes = [p, sz, p]
    lib.adatopk_wire_parse_header.restype = i32
    lib.adatopk_compress_wire.argtypes = [p, i64, i32, i64, i32, ctypes.c_double, p, sz, p, sz, p]
    lib.adatopk_compress_wire.restype = i32
    lib.adatopk_compress_wire_segmented.argtypes = [p, p, p, i32, i32, i32, p, p, p, sz, p, sz, p]
    lib.adatopk_compress_wire_segmented.restype = i32
    lib.adatopk_decompress_wire.argtypes = [p, sz, i32, i32, i64, i32, p, p]
    lib.adatopk_decompress_wire.restype = i32
    lib.adatopk_compress_segmented.argtypes = [p, p, p, i32, i32, p, p, p, p, p, sz, p]
    lib.adatopk_compress_segmented.restype = i32
    lib.adatopk_adaptive_ratios.argtypes = [p, i32, ctypes.c_double, ctypes.c_double, p]
    lib.adatopk_adaptive_ratios.restype = i32
    lib.adatopk_k_for_ratio.argtypes = [i64, ctypes.c_double]
    lib.adatopk_k_for_ratio.restype = i64
    dbl = ctypes.c_double
    lib.adatopk_link_time.argtypes = [dbl, dbl, dbl]
    lib.adatopk_link_time.restype = dbl
    lib.adatopk_pipeline_time.argtypes = [p, p, i32, i32]
    lib.adatopk_pipeline_time.restype = dbl
    lib.adatopk_pipeline_time_compressed.argtypes = [p, p, i32, i32, dbl, dbl, i32]
    lib.adatopk_pipeline_time_compressed.restype = dbl
    lib.adatopk_plan_keep_counts.argtypes = [p, p, p, i32, i32, dbl, dbl, p, p]
    lib.adatopk_plan_keep_counts.restype = i32
    lib.adatopk_compress_noalloc.argtypes = [p, i64, i32, i64, p, p, p, p]
    lib.adatopk_compress_noalloc.restype = i32
    return lib


def _check(status: int, where: str) -> None:
    if status != OK:
        raise AdaTopKError(status, where)


def _dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return F32
    if t == torch.bfloat16:
        return BF16
    if t == torch.float16:
        return F16
    raise TypeError("adatopk supports float32, bfloat16 and float16 tensors, got %s" % t)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor) -> int:
    if not (t.is_cuda and t.is_contiguous()):
        raise ValueError("adatopk needs contiguous device tensors")
    return t.data_ptr()


def _dev_or_pinned(t: torch.Tensor) -> int:
    """Device tensor, or pinned host memory (which the device addresses directly: the kernels then write over the bus)."""
    if t.is_contiguous() and (t.is_cuda or t.is_pinned()):
        return t.data_ptr()
    raise ValueError("adatopk needs a contiguous device tensor or pinned host tensor here")


def _check_outputs(dtype: torch.dtype, k_total: int, idx_out: torch.Tensor, val_out: torch.Tensor,
                   err_norm_out: Optional[torch.Tensor], num_tensors: int) -> None:
    """Output buffers of a compress call: the library gets raw pointers and cannot see their sizes or
    types, so a buffer that is too small or of another type is refused here."""
    if idx_out.dtype != torch.int32 or idx_out.numel() < k_total:
        raise ValueError("idx_out must be int32 with at least %d entries" % k_total)
    if val_out.dtype != dtype or val_out.numel() < k_total:
        raise ValueError("val_out must have the dense tensor's dtype (%s) and at least %d entries" % (dtype, k_total))
    if err_norm_out is not None and (err_norm_out.dtype != torch.float32 or err_norm_out.numel() < num_tensors):
        raise ValueError("err_norm_out must be float32 with one entry per tensor (%d)" % num_tensors)


def _check_pairs(dtype: torch.dtype, k_total: int, idx: torch.Tensor, val: torch.Tensor) -> None:
    if idx.dtype != torch.int32 or idx.numel() < k_total:
        raise ValueError("idx must be int32 with at least %d entries" % k_total)
    if val.dtype != dtype or val.numel() < k_total:
        raise ValueError("val must have the dense tensor's dtype (%s) and at least %d entries" % (dtype, k_total))


def _one_dtype(tensors: Sequence[torch.Tensor]) -> None:
    if any(t.dtype != tensors[0].dtype for t in tensors):
        raise ValueError("all tensors of a segmented call must share one dtype")


def adatopk_workspace_bytes(n_total: int, num_segments: int, dtype: torch.dtype) -> int:
    return int(load_library().adatopk_workspace_bytes(int(n_total), int(num_segments), _dtype_code(dtype)))


def new_workspace(n_total: int, num_segments: int, dtype: torch.dtype, device="cuda") -> torch.Tensor:
    nbytes = adatopk_workspace_bytes(n_total, num_segments, dtype)
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def adatopk_compress(dense: torch.Tensor, k: int, idx_out: torch.Tensor, val_out: torch.Tensor,
                     err_norm_out: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    """Enqueues compress of one tensor on the current stream; outputs are written in place."""
    lib = load_library()
    _check_outputs(dense.dtype, int(k), idx_out, val_out, err_norm_out, 1)
    err_ptr = _dev(err_norm_out) if err_norm_out is not None else None
    _check(lib.adatopk_compress(_dev(dense), dense.numel(), _dtype_code(dense.dtype), int(k), _dev(idx_out),
                                _dev(val_out), err_ptr, _dev(workspace), workspace.numel(), _stream()),
           "adatopk_compress")


def adatopk_compress_noalloc(dense: torch.Tensor, k: int, idx_out: torch.Tensor, val_out: torch.Tensor,
                             err_norm_out: Optional[torch.Tensor]) -> None:
    """adatopk_compress on the library's own resident scratch (no workspace argument, nothing allocated)."""
    lib = load_library()
    _check_outputs(dense.dtype, int(k), idx_out, val_out, err_norm_out, 1)
    err_ptr = _dev(err_norm_out) if err_norm_out is not None else None
    _check(lib.adatopk_compress_noalloc(_dev(dense), dense.numel(), _dtype_code(dense.dtype), int(k), _dev(idx_out),
                                        _dev(val_out), err_ptr, _stream()), "adatopk_compress_noalloc")


def adatopk_decompress(idx: torch.Tensor, val: torch.Tensor, k: int, dense_out: torch.Tensor) -> None:
    lib = load_library()
    _check_pairs(dense_out.dtype, int(k), idx, val)
    _check(lib.adatopk_decompress(_dev(idx), _dev(val), int(k), _dtype_code(dense_out.dtype), _dev(dense_out),
                                  dense_out.numel(), _stream()), "adatopk_decompress")


def adatopk_decompress_sorted(idx: torch.Tensor, val: torch.Tensor, k: int, dense_out: torch.Tensor) -> None:
    """Decompress for strictly ascending idx (what adatopk_compress produces)."""
    lib = load_library()
    _check_pairs(dense_out.dtype, int(k), idx, val)
    _check(lib.adatopk_decompress_sorted(_dev(idx), _dev(val), int(k), _dtype_code(dense_out.dtype),
                                         _dev(dense_out), dense_out.numel(), _stream()), "adatopk_decompress_sorted")


def adatopk_decompress_accumulate(idx: torch.Tensor, val: torch.Tensor, k: int, dense_inout: torch.Tensor) -> None:
    """dense_inout[idx[j]] += val[j] for unique indices; every other entry is left alone."""
    lib = load_library()
    _check_pairs(dense_inout.dtype, int(k), idx, val)
    _check(lib.adatopk_decompress_accumulate(_dev(idx), _dev(val), int(k), _dtype_code(dense_inout.dtype),
                                             _dev(dense_inout), dense_inout.numel(), _stream()),
           "adatopk_decompress_accumulate")


def adatopk_decompress_segmented(idx: torch.Tensor, val: torch.Tensor, out_offset: Sequence[int],
                                 dense_out: Sequence[torch.Tensor]) -> None:
    """Decompress of S tensors from the concatenated, per-tensor ascending pairs in few launches."""
    lib = load_library()
    S = len(dense_out)
    dt = _dtype_code(dense_out[0].dtype) if S else F32
    if S:
        _one_dtype(dense_out)
        _check_pairs(dense_out[0].dtype, int(out_offset[S]), idx, val)
    ptrs = (ctypes.c_void_p * max(S, 1))(*[_dev(t) for t in dense_out])
    ns = (ctypes.c_int64 * max(S, 1))(*[t.numel() for t in dense_out])
    off = (ctypes.c_int64 * (S + 1))(*[int(v) for v in out_offset])
    _check(lib.adatopk_decompress_segmented(_dev(idx), _dev(val), off, S, dt, ptrs, ns, _stream()),
           "adatopk_decompress_segmented")


class WireHeader(ctypes.Structure):
    """Mirror of adatopk_wire_header (64 bytes)."""
    _fields_ = [("magic", ctypes.c_uint32), ("version", ctypes.c_uint16), ("algorithm", ctypes.c_uint8),
                ("dtype", ctypes.c_uint8), ("index_bytes", ctypes.c_uint8), ("reserved0", ctypes.c_uint8 * 3),
                ("err_norm", ctypes.c_float), ("n", ctypes.c_int64), ("k", ctypes.c_int64),
                ("ratio", ctypes.c_double), ("idx_offset", ctypes.c_int64), ("val_offset", ctypes.c_int64),
                ("reserved1", ctypes.c_uint8 * 8)]


def adatopk_wire_bytes(k: int, dtype_code: int, index_bytes: int) -> int:
    return int(load_library().adatopk_wire_bytes(int(k), int(dtype_code), int(index_bytes)))


def adatopk_wire_keep_count(wire_bytes: int, dtype_code: int, index_bytes: int) -> int:
    return int(load_library().adatopk_wire_keep_count(int(wire_bytes), int(dtype_code), int(index_bytes)))


def adatopk_wire_parse_header(host_bytes: bytes, wire_bytes: int) -> WireHeader:
    """Checks the first 64 bytes of a message held in host memory; raises AdaTopKError if they do not fit."""
    h = WireHeader()
    buf = ctypes.create_string_buffer(bytes(host_bytes[:64]), 64) if len(host_bytes) >= 64 else None
    _check(load_library().adatopk_wire_parse_header(buf, int(wire_bytes), ctypes.byref(h)), "adatopk_wire_parse_header")
    return h


def adatopk_compress_wire(dense: torch.Tensor, k: int, index_bytes: int, ratio: float, wire_out: torch.Tensor,
                          workspace: torch.Tensor) -> None:
    """adatopk_compress writing one wire message into the uint8 tensor wire_out (device memory, or pinned
    host memory: the message then needs no copy before the host can send it)."""
    lib = load_library()
    _check(lib.adatopk_compress_wire(_dev(dense), dense.numel(), _dtype_code(dense.dtype), int(k), int(index_bytes),
                                     float(ratio), _dev_or_pinned(wire_out), wire_out.numel() * wire_out.element_size(),
                                     _dev(workspace), workspace.numel(), _stream()), "adatopk_compress_wire")


def adatopk_compress_wire_segmented(dense: Sequence[torch.Tensor], ks: Sequence[int], index_bytes: int,
                                    ratios: Optional[Sequence[float]], wire_out: torch.Tensor,
                                    wire_offset: Sequence[int], workspace: torch.Tensor) -> None:
    """One wire message per tensor, message s at byte wire_offset[s] of the uint8 tensor wire_out."""
    lib = load_library()
    S = len(dense)
    dt = _dtype_code(dense[0].dtype) if S else F32
    if S:
        _one_dtype(dense)
    ptrs = (ctypes.c_void_p * max(S, 1))(*[_dev(t) for t in dense])
    ns = (ctypes.c_int64 * max(S, 1))(*[t.numel() for t in dense])
    kk = (ctypes.c_int64 * max(S, 1))(*[int(v) for v in ks])
    off = (ctypes.c_int64 * max(S, 1))(*[int(v) for v in wire_offset])
    rr = _dbl_array(ratios) if ratios is not None else None
    _check(lib.adatopk_compress_wire_segmented(ptrs, ns, kk, S, dt, int(index_bytes), rr, _dev_or_pinned(wire_out), off,
                                               wire_out.numel() * wire_out.element_size(), _dev(workspace),
                                               workspace.numel(), _stream()), "adatopk_compress_wire_segmented")


def adatopk_decompress_wire(wire: torch.Tensor, wire_bytes: int, index_bytes: int, dense: torch.Tensor,
                            accumulate: bool = False) -> None:
    lib = load_library()
    _check(lib.adatopk_decompress_wire(_dev(wire), int(wire_bytes), _dtype_code(dense.dtype), int(index_bytes),
                                       dense.numel(), 1 if accumulate else 0, _dev(dense), _stream()),
           "adatopk_decompress_wire")


def adatopk_compress_segmented(dense: Sequence[torch.Tensor], ks: Sequence[int], idx_out: torch.Tensor,
                               val_out: torch.Tensor, out_offset: Sequence[int],
                               err_norm_out: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    lib = load_library()
    S = len(dense)
    dt = _dtype_code(dense[0].dtype) if S else F32
    if S:
        _one_dtype(dense)
        _check_outputs(dense[0].dtype, sum(int(v) for v in ks), idx_out, val_out, err_norm_out, S)
    ptrs = (ctypes.c_void_p * max(S, 1))(*[_dev(t) for t in dense])
    ns = (ctypes.c_int64 * max(S, 1))(*[t.numel() for t in dense])
    kk = (ctypes.c_int64 * max(S, 1))(*[int(v) for v in ks])
    off = (ctypes.c_int64 * (S + 1))(*[int(v) for v in out_offset])
    err_ptr = _dev(err_norm_out) if err_norm_out is not None else None
    _check(lib.adatopk_compress_segmented(ptrs, ns, kk, S, dt, _dev(idx_out), _dev(val_out), off, err_ptr,
                                          _dev(workspace), workspace.numel(), _stream()),
           "adatopk_compress_segmented")


def adatopk_adaptive_ratios(R: Sequence[float], r_user: float, coeff: float = 3.0):
    lib = load_library()
    m = len(R)
    arr = (ctypes.c_double * max(m, 1))(*[float(v) for v in R])
    out = (ctypes.c_double * max(m, 1))()
    _check(lib.adatopk_adaptive_ratios(arr, m, float(r_user), float(coeff), out), "adatopk_adaptive_ratios")
    return [out[i] for i in range(m)]


def adatopk_k_for_ratio(n: int, r_i: float) -> int:
    return int(load_library().adatopk_k_for_ratio(int(n), float(r_i)))


def _dbl_array(v):
    return (ctypes.c_double * max(len(v), 1))(*[float(x) for x in v])


def adatopk_link_time(alpha: float, beta: float, message_bytes: float) -> float:
    return float(load_library().adatopk_link_time(float(alpha), float(beta), float(message_bytes)))


def adatopk_pipeline_time(C: Sequence[float], R: Sequence[float], n_b: int) -> float:
    return float(load_library().adatopk_pipeline_time(_dbl_array(C), _dbl_array(R), len(C), int(n_b)))


def adatopk_pipeline_time_compressed(C: Sequence[float], R: Sequence[float], n_b: int, r_user: float,
                                     coeff: float = 3.0, variant: int = 0) -> float:
    return float(load_library().adatopk_pipeline_time_compressed(_dbl_array(C), _dbl_array(R), len(C), int(n_b),
                                                                 float(r_user), float(coeff), int(variant)))


def adatopk_plan_keep_counts(alpha: Sequence[float], beta: Sequence[float], n: Sequence[int], dtype_code: int,
                             r_user: float, coeff: float = 3.0):
    """(ratios, keep counts) for tensors of n[s] values crossing links (alpha[s], beta[s])."""
    m = len(n)
    ns = (ctypes.c_int64 * max(m, 1))(*[int(v) for v in n])
    r_out = (ctypes.c_double * max(m, 1))()
    k_out = (ctypes.c_int64 * max(m, 1))()
    _check(load_library().adatopk_plan_keep_counts(_dbl_array(alpha), _dbl_array(beta), ns, m, int(dtype_code),
                                                   float(r_user), float(coeff), r_out, k_out),
           "adatopk_plan_keep_counts")
    return [r_out[i] for i in range(m)], [int(k_out[i]) for i in range(m)]


# ------------------------------------------------------------------ measurement hooks (measuring build only)
def measure_stage_names():
    lib = load_measure_library()
    return [lib.adatopk_measure_stage_name(i).decode() for i in range(lib.adatopk_measure_stage_count())]


def measure_read():
    lib = load_measure_library()
    n = lib.adatopk_measure_stage_count()
    buf = (ctypes.c_float * n)()
    _check(lib.adatopk_measure_read(buf), "adatopk_measure_read")
    return [buf[i] for i in range(n)]


def measure_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    _check(load_measure_library().adatopk_measure_copy(_dev(dst), _dev(src), nbytes, _stream()), "adatopk_measure_copy")


def measure_read_only(src: torch.Tensor, sink: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    _check(load_measure_library().adatopk_measure_read_only(_dev(src), nbytes, _dev(sink), _stream()),
           "adatopk_measure_read_only")


def measure_fill(dst: torch.Tensor) -> None:
    nbytes = dst.numel() * dst.element_size()
    _check(load_measure_library().adatopk_measure_fill(_dev(dst), nbytes, _stream()), "adatopk_measure_fill")
