"""adatopk_compress_noalloc (the compress call for callers that cannot allocate: its scratch is an array
resident in the library's device image) against adatopk_compress, which takes the same scratch as a
caller-provided workspace: two calls in a row through the C ABI, the second on a smaller tensor, so that
whatever the first call left in the shared array would show."""
import numpy as np
import pytest

from paper_2410_12707_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _both(x, k):
    import torch

    import gpu_harness as H
    from paper_2410_12707_amd import binding as B

    d = H.to_device(x)
    outs = []
    for noalloc in (True, False):
        idx = torch.full((max(k, 1),), -7, dtype=torch.int32, device="cuda")
        val = torch.zeros(max(k, 1), dtype=d.dtype, device="cuda")
        err = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
        if noalloc:
            B.adatopk_compress_noalloc(d, k, idx, val, err)
        else:
            B.adatopk_compress(d, k, idx, val, err, B.new_workspace(d.numel(), 1, d.dtype))
        torch.cuda.synchronize()
        outs.append((H.to_host(idx)[:k], H.to_host(val)[:k], H.to_host(err)[0]))
    return outs


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_noalloc_matches_the_workspace_call_twice_in_a_row(dtype):
    import gpu_harness as H
    from oracle import adatopk_oracle as orc

    # first a tensor that takes the multi-kernel path with ties at the threshold, then a smaller one (and
    # one small enough for the one-workgroup path), all through the same resident array
    for n, k, kind in ((3_000_017, 30_000, "few_levels"), (1_200_003, 12_000, "normal"), (70_001, 700, "normal"),
                       (5_000, 50, "normal"), (0, 0, "normal")):
        x = wl.small_case(kind, n, seed=n + 5, dtype=dtype) if n else wl.small_case(kind, 1, 1, dtype=dtype)[:0]
        (ai, av, ae), (bi, bv, be) = _both(x, k)
        assert np.array_equal(ai, bi) and np.array_equal(H.bits(av), H.bits(bv)), (dtype, n, k)
        assert np.float32(ae).view(np.uint32) == np.float32(be).view(np.uint32), (dtype, n, k, ae, be)
        ri, rv, re = orc.compress(x, k)  # and both are the oracle's result
        assert np.array_equal(ai, ri) and np.array_equal(H.bits(av), H.bits(rv)) and H.same_err(ae, re), (dtype, n, k)


def test_noalloc_refuses_what_does_not_fit():
    import torch

    from paper_2410_12707_amd import binding as B

    n = 8_000_000  # the smallest tensor (in steps of doubling) whose scratch is beyond the resident array
    while B.adatopk_workspace_bytes(n, 1, torch.float32) <= 64 << 20:
        n *= 2
    assert n <= 512_000_000
    x = torch.zeros(n, device="cuda")
    idx = torch.zeros(10, dtype=torch.int32, device="cuda")
    val = torch.zeros(10, device="cuda")
    with pytest.raises(B.AdaTopKError) as e:
        B.adatopk_compress_noalloc(x, 10, idx, val, None)
    assert e.value.status == B.EWORKSPACE
