"""Wire messages on the GPU: compress straight into the message layout (int32 and int64 indices),
decompress and accumulate straight out of it; byte for byte against the oracle's packing."""
import struct

import numpy as np
import pytest

from oracle import adatopk_oracle as orc
from oracle import wire_format as wf
from paper_2410_12707_amd import workloads as wl

pytestmark = pytest.mark.gpu

ERR_RTOL = 1e-5
GUARD = 64


def gpu_message(x, k, ib, ratio):
    import torch

    import gpu_harness as H
    from paper_2410_12707_amd import binding as B

    d = H.to_device(x)
    nbytes = wf.message_bytes(k, x.dtype, ib)
    buf = torch.full((nbytes + GUARD,), 0xAB, dtype=torch.uint8, device="cuda")
    ws = B.new_workspace(d.numel(), 1, d.dtype)
    B.adatopk_compress_wire(d, k, ib, ratio, buf[:nbytes], ws)
    torch.cuda.synchronize()
    raw = buf.cpu().numpy().tobytes()
    assert raw[nbytes:] == b"\xAB" * GUARD, "wrote past the message"
    return raw[:nbytes]


@pytest.mark.parametrize("ib", [4, 8])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_compress_wire_is_the_oracle_message(dtype, ib):
    import gpu_harness as H

    for n, k, kind in ((1, 1, "normal"), (1000, 0, "normal"), (1000, 7, "few_levels"), (70_001, 701, "normal"),
                       (3_300_017, 33_001, "normal"), (250_000, 250_000, "sparse")):
        x = wl.small_case(kind, n, seed=n + k, dtype=dtype)
        ri, rv, re = orc.compress(x, k)
        ref = wf.pack(ri, rv, n, float(re), 100.0, ib)
        got = gpu_message(x, k, ib, 100.0)
        assert len(got) == len(ref)
        assert got[:12] == ref[:12] and got[16:] == ref[16:], (dtype, ib, n, k)
        assert H.same_err(struct.unpack("<f", got[12:16])[0], re, ERR_RTOL)
        hdr, gi, gv = wf.unpack(got)
        assert hdr["k"] == k and np.array_equal(gi, ri.astype(np.int64))


@pytest.mark.parametrize("ib", [4, 8])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_decompress_wire_overwrite_and_accumulate(dtype, ib):
    import torch

    import gpu_harness as H
    from paper_2410_12707_amd import binding as B

    for n, k in ((1, 1), (1000, 0), (70_001, 701), (2_000_003, 150_000), (2_000_003, 20_000)):
        x = wl.small_case("normal", n, seed=3 * n + k, dtype=dtype)
        ri, rv, re = orc.compress(x, k)
        msg = wf.pack(ri, rv, n, float(re), 50.0, ib)  # the oracle's message, uploaded as a receiver would
        dev = torch.from_numpy(np.frombuffer(msg, dtype=np.uint8).copy()).cuda()
        base = wl.small_case("normal", n, seed=17, dtype=dtype)
        y = H.to_device(base)
        B.adatopk_decompress_wire(dev, len(msg), ib, y, accumulate=True)
        torch.cuda.synchronize()
        assert np.array_equal(H.bits(H.to_host(y)), H.bits(orc.decompress_accumulate(ri, rv, base))), (dtype, ib, n, k)
        B.adatopk_decompress_wire(dev, len(msg), ib, y, accumulate=False)
        torch.cuda.synchronize()
        assert np.array_equal(H.bits(H.to_host(y)), H.bits(orc.decompress(ri, rv, n))), (dtype, ib, n, k)


def test_wire_round_trip_on_the_device_config1():
    # GPU message -> GPU decompress, the whole path a sender / receiver pair runs, at a benchmark shape
    import torch

    import gpu_harness as H
    from paper_2410_12707_amd import binding as B

    w = wl.config1()
    x, k = w.tensors[0], w.ks[0]
    for ib in (4, 8):
        msg = gpu_message(x, k, ib, 100.0)
        h = B.adatopk_wire_parse_header(msg, len(msg))
        assert (h.n, h.k, h.index_bytes) == (x.size, k, ib)
        dev = torch.from_numpy(np.frombuffer(msg, dtype=np.uint8).copy()).cuda()
        y = torch.empty(x.size, dtype=torch.float32, device="cuda")
        B.adatopk_decompress_wire(dev, len(msg), ib, y)
        torch.cuda.synchronize()
        ri, rv, _ = orc.compress(x, k)
        assert np.array_equal(H.bits(H.to_host(y)), H.bits(orc.decompress(ri, rv, x.size)))
