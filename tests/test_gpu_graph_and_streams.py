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


def test_host_threads_each_with_a_stream_and_a_workspace():
    # The library keeps no state between calls, so host threads may call it at the same time as long
    # as each brings its own workspace and outputs (ctypes drops the interpreter lock during a call,
    # so the calls really do overlap in the library's host code).
    import threading

    import torch

    from paper_2410_12707_amd import binding as B

    kinds = ["normal", "few_levels", "all_equal", "sparse"]
    sizes = [300_001, 70_000, 8_192, 1_234_567]
    jobs = [(wl.small_case(kind, n, seed=40 + t), max(1, n // (50 * (t + 1)))) for t, (kind, n) in enumerate(zip(kinds, sizes))]
    results, failures = [None] * len(jobs), []

    def worker(t):
        try:
            x, k = jobs[t]
            n = x.size
            st = torch.cuda.Stream()
            with torch.cuda.stream(st):
                d = torch.from_numpy(x).cuda()
                idx = torch.empty(k, dtype=torch.int32, device="cuda")
                val = torch.empty(k, dtype=torch.float32, device="cuda")
                err = torch.empty(1, dtype=torch.float32, device="cuda")
                y = torch.empty(n, dtype=torch.float32, device="cuda")
                ws = B.new_workspace(n, 1, torch.float32)
                for _ in range(25):
                    B.adatopk_compress(d, k, idx, val, err, ws)
                    B.adatopk_decompress_sorted(idx, val, k, y)
                st.synchronize()
                results[t] = (idx.cpu().numpy(), val.cpu().numpy(), float(err.cpu()[0]), y.cpu().numpy())
        except Exception as e:  # reported by the main thread
            failures.append((t, repr(e)))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(len(jobs))]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not failures, failures
    for (x, k), (gi, gv, ge, gy) in zip(jobs, results):
        ri, rv, re = orc.compress(x, k)
        assert np.array_equal(gi, ri)
        assert np.array_equal(gv.view(np.uint32), rv.view(np.uint32))
        assert abs(ge - float(re)) <= 1e-5 * max(float(re), 1e-30)
        assert np.array_equal(gy.view(np.uint32), orc.decompress(ri, rv, x.size).view(np.uint32))


def test_micro_batch_pipeline_overlapping_compress_and_message_copy():
    # Sender side of pipeline parallelism with several micro-batches (paper Sec. 3.6): micro-batch j + 1
    # is compressed into a wire message while the message of micro-batch j is copied to pinned host
    # memory on a second stream; two message buffers, events in both directions.  Every message that
    # arrives on the host must be the oracle's message of that micro-batch; the receiver side
    # (upload, accumulate into a running gradient) must give the oracle's sum.
    import struct

    import torch

    import gpu_harness as H
    from oracle import wire_format as wf
    from paper_2410_12707_amd import binding as B

    n, k, n_b = 600_011, 6_000, 5
    xs = [wl.small_case(kind, n, seed=300 + j) for j, kind in enumerate(["normal", "few_levels", "sparse", "normal", "normal"])]
    refs = [orc.compress(x, k) for x in xs]
    dev = [H.to_device(x) for x in xs]
    nbytes = wf.message_bytes(k, np.float32, 4)
    wire = [torch.full((nbytes,), 0xEE, dtype=torch.uint8, device="cuda") for _ in range(2)]
    host = [torch.empty(nbytes, dtype=torch.uint8, pin_memory=True) for _ in range(n_b)]
    ws = B.new_workspace(n, 1, torch.float32)
    comp, copy = torch.cuda.Stream(), torch.cuda.Stream()
    done = [torch.cuda.Event() for _ in range(2)]
    freed = [torch.cuda.Event() for _ in range(2)]
    torch.cuda.synchronize()
    for e in freed:
        e.record(comp)
    for j in range(n_b):
        b = j % 2
        with torch.cuda.stream(comp):
            comp.wait_event(freed[b])
            B.adatopk_compress_wire(dev[j], k, 4, n / k, wire[b], ws)
            done[b].record(comp)
        with torch.cuda.stream(copy):
            copy.wait_event(done[b])
            host[j].copy_(wire[b], non_blocking=True)
            freed[b].record(copy)
    torch.cuda.synchronize()
    acc_ref = np.zeros(n, dtype=np.float32)
    acc = torch.zeros(n, dtype=torch.float32, device="cuda")
    for j in range(n_b):
        ri, rv, re = refs[j]
        got = host[j].numpy().tobytes()
        ref = wf.pack(ri, rv, n, float(re), n / k, 4)
        assert got[:12] == ref[:12] and got[16:] == ref[16:], j
        assert H.same_err(struct.unpack("<f", got[12:16])[0], re, 1e-5)
        h = B.adatopk_wire_parse_header(got, len(got))
        assert (h.n, h.k) == (n, k)
        up = host[j].cuda()  # the receiver uploads the message and adds it to its running gradient
        B.adatopk_decompress_wire(up, nbytes, 4, acc, accumulate=True)
        acc_ref = orc.decompress_accumulate(ri, rv, acc_ref)
    torch.cuda.synchronize()
    assert np.array_equal(H.bits(H.to_host(acc)), H.bits(acc_ref))


def test_measurement_hooks_do_what_the_benchmark_assumes():
    # the plain kernels that scale the hardware counters and give the streaming ceilings: the copy
    # really copies, the fill really zeroes, and the stage timers report the kernels of the last call
    import torch

    from paper_2410_12707_amd import binding as B

    n = 1_000_003
    src = torch.randn(n, device="cuda")
    dst = torch.full((n,), 7.0, device="cuda")
    B.measure_copy(dst[: n - 3], src[: n - 3])  # whole 16-byte units only
    torch.cuda.synchronize()
    assert bool((dst[: n - 3] == src[: n - 3]).all()) and bool((dst[n - 3:] == 7.0).all())
    B.measure_fill(dst[:1000])
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    B.measure_read_only(src[: n - 3], sink)
    torch.cuda.synchronize()
    assert bool((dst[:1000] == 0).all()) and float(dst[1000]) == float(src[1000])

    k = 10_000
    idx = torch.empty(k, dtype=torch.int32, device="cuda")
    val = torch.empty(k, device="cuda")
    ws = B.new_workspace(n, 1, torch.float32)
    with B.measuring():  # the measuring build of the library: the same kernels, every launch with events
        B.adatopk_compress(src, k, idx, val, None, ws)
        torch.cuda.synchronize()
        ms = dict(zip(B.measure_stage_names(), B.measure_read()))
    for name in ("k_hist1", "k_scan", "k_refine", "k_emit"):
        assert 0.0 < ms[name] < 5.0, (name, ms[name])  # milliseconds; each of these kernels takes microseconds here
    assert ms["k_merge"] < 0 and ms["k_small"] < 0  # not launched by this call
    assert ms["k_scan_spec"] < 0  # a tensor of a million elements and a bit is not worth a speculative pass


def test_graph_capture_of_wire_and_segmented_calls():
    # the wire and the segmented entry points enqueue kernels only as well: captured once, replayed on new data
    import struct

    import torch

    import gpu_harness as H
    from oracle import wire_format as wf
    from paper_2410_12707_amd import binding as B

    lens = [40_000, 3_000, 150_000]
    ks = [400, 300, 15_000]
    cases = [[wl.small_case(kind, n, seed=s * 10 + i) for i, n in enumerate(lens)]
             for s, kind in enumerate(["normal", "few_levels", "sparse"])]
    ds = [torch.empty(n, dtype=torch.float32, device="cuda") for n in lens]
    offs, pos = [], 0
    for k in ks:
        offs.append(pos)
        pos += (wf.message_bytes(k, np.float32, 8) + 15) // 16 * 16
    wire = torch.zeros(pos, dtype=torch.uint8, device="cuda")
    ys = [torch.empty(n, dtype=torch.float32, device="cuda") for n in lens]
    ws = B.new_workspace(sum(lens), len(lens), torch.float32)

    def enqueue():
        B.adatopk_compress_wire_segmented(ds, ks, 8, None, wire, offs, ws)
        for s, (n, k) in enumerate(zip(lens, ks)):
            nb = wf.message_bytes(k, np.float32, 8)
            B.adatopk_decompress_wire(wire[offs[s]:offs[s] + nb], nb, 8, ys[s])

    for d, x in zip(ds, cases[0]):
        d.copy_(torch.from_numpy(x))
    enqueue()  # eager warm-up
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        enqueue()
    for rep in range(5):
        xs = cases[rep % 3]
        for d, x in zip(ds, xs):
            d.copy_(torch.from_numpy(x))
        wire.zero_()
        g.replay()
        torch.cuda.synchronize()
        raw = wire.cpu().numpy().tobytes()
        for s, (x, k) in enumerate(zip(xs, ks)):
            ri, rv, re = orc.compress(x, k)
            ref = wf.pack(ri, rv, lens[s], float(re), lens[s] / k, 8)
            got = raw[offs[s]:offs[s] + len(ref)]
            assert got[:12] == ref[:12] and got[16:] == ref[16:], (rep, s)
            assert H.same_err(struct.unpack("<f", got[12:16])[0], re, 1e-5)
            assert np.array_equal(H.bits(H.to_host(ys[s])), H.bits(orc.decompress(ri, rv, lens[s]))), (rep, s)
