"""CPU statement of the wire message layout (TEST INFRASTRUCTURE, like the rest of ``oracle/``).

The message is the (index, value) pairs of the paper's Sec. 5.1 behind a 64-byte header holding
what the paper's message descriptor keeps for compression (Compress_cfg, Sec. 3.4).  This module
writes and reads it field by field with ``struct`` from the documented byte offsets; it shares no
declaration with the product library.

    offset  size  field
    0       4     magic        0x314B5441 ("ATK1"), little-endian like every field
    4       2     version      1
    6       1     algorithm    1 = top-k by magnitude
    7       1     dtype        0 fp32, 1 bf16, 2 fp16
    8       1     index_bytes  4 or 8
    9       3     zero
    12      4     err_norm     float32
    16      8     n            int64
    24      8     k            int64
    32      8     ratio        float64
    40      8     idx_offset   int64 = 64
    48      8     val_offset   int64 = 64 + k * index_bytes rounded up to a multiple of 16
    56      8     zero
    64            k indices (ascending), zero padding to val_offset, k values
"""
from __future__ import annotations

import struct

import numpy as np

HEADER_BYTES = 64
_FMT = "<IHBBB3xfqqdqq8x"
assert struct.calcsize(_FMT) == HEADER_BYTES

_DTYPE_CODE = {np.dtype(np.float32): 0, np.dtype(np.uint16): 1, np.dtype(np.float16): 2}
_CODE_DTYPE = {v: k for k, v in _DTYPE_CODE.items()}


def value_offset(k: int, index_bytes: int) -> int:
    return HEADER_BYTES + (k * index_bytes + 15) // 16 * 16


def message_bytes(k: int, value_dtype, index_bytes: int) -> int:
    return value_offset(k, index_bytes) + k * np.dtype(value_dtype).itemsize


def pack(idx: np.ndarray, val: np.ndarray, n: int, err_norm: float, ratio: float, index_bytes: int) -> bytes:
    """Bytes of the message for the pairs (idx, val) of a tensor of n elements."""
    k = int(idx.size)
    assert val.size == k and index_bytes in (4, 8)
    voff = value_offset(k, index_bytes)
    head = struct.pack(_FMT, 0x314B5441, 1, 1, _DTYPE_CODE[val.dtype], index_bytes, float(err_norm), int(n), k,
                       float(ratio), HEADER_BYTES, voff)
    body = np.ascontiguousarray(idx, dtype="<i4" if index_bytes == 4 else "<i8").tobytes()
    body += b"\x00" * (voff - HEADER_BYTES - len(body))
    return head + body + np.ascontiguousarray(val).tobytes()


def unpack(msg: bytes):
    """(header dict, idx int64 array, val array) of a message; raises ValueError if it is malformed."""
    if len(msg) < HEADER_BYTES:
        raise ValueError("shorter than a header")
    magic, version, algo, dt, ib, err, n, k, ratio, ioff, voff = struct.unpack(_FMT, msg[:HEADER_BYTES])
    if magic != 0x314B5441 or version != 1 or algo != 1 or dt not in _CODE_DTYPE or ib not in (4, 8):
        raise ValueError("bad header")
    vdt = _CODE_DTYPE[dt]
    if not (0 <= k <= n) or ioff != HEADER_BYTES or voff != value_offset(k, ib) or len(msg) != message_bytes(k, vdt, ib):
        raise ValueError("sizes do not fit")
    idx = np.frombuffer(msg, dtype="<i4" if ib == 4 else "<i8", count=k, offset=ioff).astype(np.int64)
    val = np.frombuffer(msg, dtype=vdt, count=k, offset=voff).copy()
    hdr = dict(dtype=vdt, index_bytes=ib, err_norm=err, n=n, k=k, ratio=ratio, idx_offset=ioff, val_offset=voff)
    return hdr, idx, val
