"""The wire message: the oracle's byte layout pinned by hand-worked bytes and by the sizes the paper
prints; the library's host-side size / header routines checked against it (CPU only)."""
import json
import os
import struct

import numpy as np
import pytest

from oracle import wire_format as wf
from paper_2410_12707_amd import binding as B

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
DT = {"f32": (np.float32, B.F32), "bf16": (np.uint16, B.BF16), "f16": (np.float16, B.F16)}


def test_hand_worked_message_bytes():
    idx = np.array([1, 4], dtype=np.int32)
    val = np.array([1.0, -2.0], dtype=np.float32)
    msg = wf.pack(idx, val, n=6, err_norm=0.5, ratio=3.0, index_bytes=4)
    assert len(msg) == 64 + 16 + 8
    assert msg[0:4] == b"ATK1" and msg[4:9] == bytes([1, 0, 1, 0, 4]) and msg[9:12] == b"\0\0\0"
    assert msg[12:16] == bytes([0, 0, 0, 0x3F])  # 0.5f
    assert msg[16:24] == bytes([6, 0, 0, 0, 0, 0, 0, 0]) and msg[24:32] == bytes([2, 0, 0, 0, 0, 0, 0, 0])
    assert msg[32:40] == bytes([0, 0, 0, 0, 0, 0, 0x08, 0x40])  # 3.0
    assert msg[40:48] == bytes([64, 0, 0, 0, 0, 0, 0, 0]) and msg[48:56] == bytes([80, 0, 0, 0, 0, 0, 0, 0])
    assert msg[56:64] == b"\0" * 8
    assert msg[64:72] == bytes([1, 0, 0, 0, 4, 0, 0, 0]) and msg[72:80] == b"\0" * 8
    assert msg[80:88] == bytes([0, 0, 0x80, 0x3F, 0, 0, 0, 0xC0])
    wide = wf.pack(idx, val, n=6, err_norm=0.5, ratio=3.0, index_bytes=8)
    assert len(wide) == 64 + 16 + 8 and wide[8] == 8
    assert wide[64:80] == bytes([1, 0, 0, 0, 0, 0, 0, 0, 4, 0, 0, 0, 0, 0, 0, 0])


def test_hand_worked_sizes_and_the_papers_accounting():
    assert wf.message_bytes(0, np.float32, 4) == 64
    assert wf.message_bytes(3, np.float32, 4) == 64 + 16 + 12
    assert wf.message_bytes(3, np.float32, 8) == 64 + 32 + 12
    assert wf.message_bytes(5, np.uint16, 4) == 64 + 32 + 10
    with open(os.path.join(GOLDEN, "wire_size.json")) as f:
        g = json.load(f)
    # fp32 values with int64 indices at ratio 100: the paper prints 33.3x less data than the dense tensor
    n = 25_165_824
    k = n // g["ratio"]
    pairs = wf.message_bytes(k, np.float32, 8) - wf.HEADER_BYTES
    assert abs(n * 4 / pairs - g["latency_fig_shrink_at_ratio_100"]) < 0.05
    assert pairs // k == 4 * g["adacompress_coefficient"]  # 12 bytes per pair = 3 x the value alone


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("ib", [4, 8])
def test_round_trip_and_library_host_routines(dtype, ib):
    npdt, code = DT[dtype]
    rng = np.random.Generator(np.random.PCG64(3))
    for k in (0, 1, 2, 3, 4, 5, 7, 8, 1000, 4097):
        n = 3 * k + 5
        idx = np.sort(rng.permutation(n)[:k]).astype(np.int32)
        val = rng.integers(0, 1 << 16, size=k).astype(np.uint16).view(npdt) if npdt != np.float32 else \
            rng.standard_normal(k).astype(np.float32)
        msg = wf.pack(idx, val, n, err_norm=1.25, ratio=100.0, index_bytes=ib)
        hdr, i2, v2 = wf.unpack(msg)
        assert np.array_equal(i2, idx) and np.array_equal(v2.view(np.uint8), val.view(np.uint8))
        assert (hdr["n"], hdr["k"], hdr["ratio"], hdr["err_norm"]) == (n, k, 100.0, 1.25)
        assert B.adatopk_wire_bytes(k, code, ib) == len(msg)
        assert B.adatopk_wire_keep_count(len(msg), code, ib) == k
        h = B.adatopk_wire_parse_header(msg, len(msg))
        assert (h.n, h.k, h.dtype, h.index_bytes, h.ratio, h.err_norm) == (n, k, code, ib, 100.0, 1.25)
        assert (h.idx_offset, h.val_offset) == (hdr["idx_offset"], hdr["val_offset"])


def test_library_rejects_sizes_and_headers_that_do_not_fit():
    assert B.adatopk_wire_bytes(-1, B.F32, 4) == 0 and B.adatopk_wire_bytes(5, 9, 4) == 0
    assert B.adatopk_wire_bytes(5, B.F32, 2) == 0 and B.adatopk_wire_bytes(1 << 31, B.F32, 4) == 0
    assert B.adatopk_wire_keep_count(63, B.F32, 4) == -1
    assert B.adatopk_wire_keep_count(64 + 16 + 12 + 1, B.F32, 4) == -1  # between k = 3 and k = 4
    sizes = {B.adatopk_wire_bytes(k, B.BF16, 4) for k in range(200)}
    for b in range(64, max(sizes) + 1):
        k = B.adatopk_wire_keep_count(b, B.BF16, 4)
        assert (k >= 0) == (b in sizes) and (k < 0 or B.adatopk_wire_bytes(k, B.BF16, 4) == b)
    good = wf.pack(np.array([0, 2], np.int32), np.array([1.0, 2.0], np.float32), 4, 0.0, 2.0, 4)
    B.adatopk_wire_parse_header(good, len(good))

    def broken(offset, fmt, value):
        b = bytearray(good)
        struct.pack_into(fmt, b, offset, value)
        return bytes(b)

    for bad in (broken(0, "<I", 0x12345678), broken(4, "<H", 2), broken(6, "<B", 7), broken(7, "<B", 5),
                broken(8, "<B", 2), broken(24, "<q", 5), broken(24, "<q", -1), broken(40, "<q", 32),
                broken(48, "<q", 96)):
        with pytest.raises(B.AdaTopKError):
            B.adatopk_wire_parse_header(bad, len(bad))
    with pytest.raises(B.AdaTopKError):
        B.adatopk_wire_parse_header(good, len(good) + 16)  # a length that belongs to another k
    with pytest.raises(ValueError):
        wf.unpack(good[:-1])
