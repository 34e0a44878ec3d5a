"""The calls only enqueue kernels: they can be captured into a HIP graph and replayed, and they
run on whatever stream is current.  Replays are checked against the eager result and the oracle."""
import numpy as np
import pytest

from oracle import adatopk_oracle as orc
from paper_2410_12707_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_graph_capture_and_replay():
    import torch

    from paper_2410_12707_amd import binding as B

    n, k = 1_000_003, 12_345
    xs = [wl.small_case(kind, n, seed=s) for s, kind in enumerate(["normal", "few_levels", "sparse"])]
    refs = [orc.compress(x, k) for x in xs]
    d = torch.empty(n, dtype=torch.float32, device="cuda")
    idx = torch.empty(k, dtype=torch.int32, device="cuda")
    val = torch.empty(k, dtype=torch.float32, device="cuda")
    err = torch.empty(1, dtype=torch.float32, device="cuda")
    y = torch.empty(n, dtype=torch.float32, device="cuda")
    ws = B.new_workspace(n, 1, torch.float32)

    d.copy_(torch.from_numpy(xs[0]))
    B.adatopk_compress(d, k, idx, val, err, ws)  # eager warm-up on the default stream
    B.adatopk_decompress_sorted(idx, val, k, y)
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.adatopk_compress(d, k, idx, val, err, ws)
        B.adatopk_decompress_sorted(idx, val, k, y)
    for rep in range(6):  # replays with eager work and synchronisation in between
        x, (ri, rv, re) = xs[rep % 3], refs[rep % 3]
        d.copy_(torch.from_numpy(x))
        idx.fill_(-1)
        y.fill_(3.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(idx.cpu().numpy(), ri), rep
        assert np.array_equal(val.cpu().numpy().view(np.uint32), rv.view(np.uint32)), rep
        assert abs(float(err.cpu()[0]) - float(re)) <= 1e-5 * float(re)
        assert np.array_equal(y.cpu().numpy().view(np.uint32), orc.decompress(ri, rv, n).view(np.uint32)), rep


def test_two_streams_with_their_own_workspaces():
    import torch

    from paper_2410_12707_amd import binding as B

    n = 2_000_003
    cases = [(wl.small_case("normal", n, seed=11), n // 100), (wl.small_case("few_levels", n, seed=12), n // 7)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = []
    for (x, k), st in zip(cases, streams):
        with torch.cuda.stream(st):
            d = torch.from_numpy(x).cuda(non_blocking=False)
            idx = torch.empty(k, dtype=torch.int32, device="cuda")
            val = torch.empty(k, dtype=torch.float32, device="cuda")
            err = torch.empty(1, dtype=torch.float32, device="cuda")
            y = torch.empty(n, dtype=torch.float32, device="cuda")
            ws = B.new_workspace(n, 1, torch.float32)
            for _ in range(3):  # several calls in flight on each stream, interleaved with the other stream's
                B.adatopk_compress(d, k, idx, val, err, ws)
                B.adatopk_decompress(idx, val, k, y)
            outs.append((d, idx, val, err, y, ws))
    torch.cuda.synchronize()
    for (x, k), (d, idx, val, err, y, ws) in zip(cases, outs):
        ri, rv, re = orc.compress(x, k)
        assert np.array_equal(idx.cpu().numpy(), ri)
        assert np.array_equal(val.cpu().numpy().view(np.uint32), rv.view(np.uint32))
        assert abs(float(err.cpu()[0]) - float(re)) <= 1e-5 * float(re)
        assert np.array_equal(y.cpu().numpy().view(np.uint32), orc.decompress(ri, rv, n).view(np.uint32))
