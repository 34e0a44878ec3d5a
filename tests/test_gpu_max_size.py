"""The largest tensor the int32 index allows (n = 2^31 - 1), checked by properties.

A full sort of two billion pairs is out of reach for the CPU oracle, so this case checks what
holds at any size and pins the result uniquely: exactly k ascending in-range indices, values equal
to the input at those indices, every kept key >= every dropped key, ties at the threshold key
resolved to the lowest indices, the error norm equal to the norm of the dropped part, and the
reconstruction equal to the masked input.  The reference quantities are computed with plain torch
ops on the device (library routines, not this repository's kernels).
"""
import math

import pytest

pytestmark = pytest.mark.gpu

N_MAX = (1 << 31) - 1


def _keys(x):
    import torch

    if x.dtype == torch.bfloat16:
        return x.view(torch.int16).to(torch.int32) & 0x7FFF
    return x.view(torch.int32) & 0x7FFFFFFF


@pytest.mark.parametrize("dtype_name,k", [("bf16", 1_000_003), ("f32", 21_474_836)])
def test_largest_index_range(dtype_name, k):
    import torch

    from paper_2410_12707_amd import binding as B

    dt = torch.bfloat16 if dtype_name == "bf16" else torch.float32
    n = N_MAX
    gen = torch.Generator(device="cuda")
    gen.manual_seed(12707)
    x = torch.empty(n, dtype=dt, device="cuda")
    step = 1 << 28
    for a in range(0, n, step):  # N(0,1) in slices, to bound the temporaries
        m = min(step, n - a)
        x[a:a + m] = torch.randn(m, generator=gen, device="cuda", dtype=torch.float32).to(dt)
    x[n - 1] = 1000.0  # the very last element must be found, at index 2^31 - 2
    x[0] = -999.0

    idx = torch.empty(k, dtype=torch.int32, device="cuda")
    val = torch.empty(k, dtype=dt, device="cuda")
    err = torch.empty(1, dtype=torch.float32, device="cuda")
    ws = B.new_workspace(n, 1, dt)
    B.adatopk_compress(x, k, idx, val, err, ws)
    torch.cuda.synchronize()
    del ws

    i64 = idx.to(torch.int64)
    assert int(i64[0]) == 0 and int(i64[-1]) == n - 1
    assert bool((i64[1:] > i64[:-1]).all())  # strictly ascending, hence unique and in range
    bits = torch.int16 if dt == torch.bfloat16 else torch.int32
    assert bool((x[i64].view(bits) == val.view(bits)).all())

    keys = _keys(x)
    mask = torch.zeros(n, dtype=torch.bool, device="cuda")
    mask[i64] = True
    assert int(mask.sum()) == k
    kept_keys = keys[i64]
    t = int(kept_keys.min())
    dropped_max = int(keys.masked_fill(mask, -1).max())
    assert t >= dropped_max
    if dropped_max == t:  # ties at the threshold: the kept ones come first
        tie_kept_last = int(i64[kept_keys == t].max())
        tie = (keys == t) & ~mask
        tie_dropped_first = int(torch.nonzero(tie[: tie_kept_last + 1]).numel())
        assert tie_dropped_first == 0
        del tie
    del keys, kept_keys

    total = 0.0
    for a in range(0, n, step):
        m = min(step, n - a)
        xs = x[a:a + m].to(torch.float64)
        total += float((xs * xs).masked_fill(mask[a:a + m], 0.0).sum())
    assert math.isclose(float(err[0]), math.sqrt(total), rel_tol=1e-5)

    y = torch.empty(n, dtype=dt, device="cuda")
    for call in (B.adatopk_decompress_sorted, B.adatopk_decompress):
        y.fill_(7.0)
        call(idx, val, k, y)
        torch.cuda.synchronize()
        expect = torch.where(mask, x, torch.zeros((), dtype=dt, device="cuda"))
        assert bool((y.view(bits) == expect.view(bits)).all())
        del expect
