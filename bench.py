#!/usr/bin/env python3
"""Benchmark of the AdaTopK hot path on one MI355X.

A step is one pass of the whole path over one tensor: adatopk_compress (threshold select,
stable compaction, error norm) followed by adatopk_decompress_sorted (zero fill + scatter of the
ascending pairs that compress wrote, one kernel), through
the C ABI, on the GPT-2-small post-GELU activation fp32 [32,1024,768] at k = 1 %.  Inputs are
resident in HBM before the timed region; the timed steps rotate over four distinct copies of
the input (403 MB, more than the 256 MB last-level cache) so that no step finds its input
cached from the step before.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE; each scaled by the
# same counter's reading for the library's plain copy kernel of known size), workload below.
# From profiles/hbm_traffic_cfg2_k1pct.md (fetched + written bytes per launch); None where no
# counter run has been made for that kernel.
TRAFFIC_BYTES = {
    "k_hist1": 100834731 + 2166848,
    "k_gather": 101826353 + 3407968,
    "k_hist3": 1805841 + 591616,
    "k_emit": 2609532 + 2021408,
    "k_merge": 6496496 + 112868013,
}


def micro_batch_pipeline(B, torch, xs, k, tdt, n, esize, ws, n_b=4, rounds=25):
    """Sender side of pipeline parallelism with n_b micro-batches (paper Sec. 3.6): every micro-batch's
    activation is compressed straight into a wire message, and the message is copied to pinned host
    memory, where a network stack would pick it up.  Serial: both on one stream.  Overlapped: the copy
    of micro-batch j runs on a second stream while the next micro-batches are compressed (n_b message buffers).
    Returns microseconds per micro-batch for both."""
    dt_code = B._dtype_code(tdt)
    nbytes = B.adatopk_wire_bytes(k, dt_code, 4)
    nbuf = n_b  # one message buffer per micro-batch in flight: a buffer is waited for only every n_b-th time
    wire = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(nbuf)]
    host = [torch.empty(nbytes, dtype=torch.uint8, pin_memory=True) for _ in range(nbuf)]
    comp, copy = torch.cuda.Stream(), torch.cuda.Stream()
    done = [torch.cuda.Event() for _ in range(nbuf)]
    freed = [torch.cuda.Event() for _ in range(nbuf)]

    def run(overlap: bool) -> float:
        torch.cuda.synchronize()
        for e in freed:
            e.record(comp)
        t0 = time.perf_counter()
        for j in range(n_b * rounds):
            b = j % nbuf
            with torch.cuda.stream(comp):
                comp.wait_event(freed[b])
                B.adatopk_compress_wire(xs[j % len(xs)][0], k, 4, float(n) / max(k, 1), wire[b], ws)
                done[b].record(comp)
            with torch.cuda.stream(copy if overlap else comp):
                if overlap:
                    copy.wait_event(done[b])
                host[b].copy_(wire[b], non_blocking=True)
                freed[b].record(copy if overlap else comp)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / (n_b * rounds) * 1e6

    def run_zero_copy() -> float:  # the kernels write the message straight into pinned host memory
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(comp):
            for j in range(n_b * rounds):
                B.adatopk_compress_wire(xs[j % len(xs)][0], k, 4, float(n) / max(k, 1), host[j % nbuf], ws)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / (n_b * rounds) * 1e6

    run(True)  # warm-up of all paths
    run_zero_copy()
    zero_copy = sorted(run_zero_copy() for _ in range(5))
    serial = sorted(run(False) for _ in range(5))
    overlapped = sorted(run(True) for _ in range(5))  # cross-stream event waits make this one vary from run to run
    return {"n_b": n_b, "message_bytes": nbytes, "serial_us_per_micro_batch": round(serial[2], 2),
            "overlapped_us_per_micro_batch": round(overlapped[2], 2),
            "overlapped_us_best_and_worst": [round(overlapped[0], 2), round(overlapped[-1], 2)],
            "into_pinned_host_us_per_micro_batch": round(zero_copy[2], 2),
            "what": "compress into a wire message + copy of the message to pinned host memory (serial: one stream; "
                    "overlapped: copies on a second stream), or the message written by the kernels straight into pinned "
                    "host memory; median of 5 runs of %d micro-batches" % (n_b * rounds)}


def concurrent_streams(B, torch, xs, k, tdt, n, esize, streams=4, rounds=50):
    """Independent compress + decompress steps on several streams, each with its own workspace and
    outputs: what the GPU sustains when the tensors of several pipeline edges are in flight at once."""
    sts = [torch.cuda.Stream() for _ in range(streams)]
    bufs = [(torch.empty(max(k, 1), dtype=torch.int32, device="cuda"), torch.empty(max(k, 1), dtype=tdt, device="cuda"),
             torch.empty(1, dtype=torch.float32, device="cuda"), torch.empty(n, dtype=tdt, device="cuda"),
             B.new_workspace(n, 1, tdt)) for _ in range(streams)]

    def run() -> float:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(rounds):
            for s_, st in enumerate(sts):
                idx, val, err, y, ws = bufs[s_]
                with torch.cuda.stream(st):
                    B.adatopk_compress(xs[(i * streams + s_) % len(xs)][0], k, idx, val, err, ws)
                    B.adatopk_decompress_sorted(idx, val, k, y)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / (rounds * streams)

    run()
    sec = run()
    return {"streams": streams, "us_per_step": round(sec * 1e6, 2), "value": round(n * esize / sec / 1e9, 1), "unit": "GB/s"}


def call_times(B, torch, compress, decompress, reps):
    """Median GPU time of the compress call and of the decompress call on their own: one pair of
    events on the launch stream around each call, `reps` calls each, inputs rotating as in the step."""
    out = {}
    for name, fn in (("t_compress_us", compress), ("t_decompress_us", decompress)):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        torch.cuda.synchronize()
        for i, (e0, e1) in enumerate(evs):
            e0.record()
            fn(i)
            e1.record()
        torch.cuda.synchronize()
        ms = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
        out[name] = round(ms[len(ms) // 2] * 1e3, 2)
    return out


def streaming_ceilings(B, torch, src, dst, reps=20):
    """What the memory system gives the library's plain kernels on a buffer of the tensor's size:
    read only, fill only, copy (GB/s of bytes moved; the copy moves twice the buffer)."""
    nbytes = src.numel() * src.element_size()
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = {}
    for name, fn, moved in (("read", lambda: B.measure_read_only(src, sink), nbytes),
                            ("fill", lambda: B.measure_fill(dst), nbytes),
                            ("copy", lambda: B.measure_copy(dst, src), 2 * nbytes)):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        fn()
        torch.cuda.synchronize()
        for e0, e1 in evs:
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        ms = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
        out[name] = round(moved / (ms[len(ms) // 2] * 1e-3) / 1e9, 1)
    out["unit"] = "GB/s"
    out["bytes"] = nbytes
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--config", default="2", choices=["1", "2a", "2", "2c", "3", "4", "5", "5h", "small", "r18"],
                    help="workload: 2 (default, the headline: GELU tensor at k = 1 %%), 2a / 2c = the same tensor at "
                         "k = 0.1 %% / 10 %%, 1, 3, 4 (segmented batch), 5 (bf16) = the other parity configurations; "
                         "5h = config 5 in fp16; small = 128 messages of 1024-8192 elements in one call, r18 = 64 "
                         "per-sample ResNet-18 stage outputs in one call (both timed as HIP graph replays: the "
                         "Python marshalling of that many pointers would otherwise be the bottleneck)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the side measurements (micro-batch pipeline, concurrent streams)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run the library's plain copy kernel on the workload-sized buffer (the known-size "
                         "kernel that hardware-counter readings are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2410_12707_amd import binding as B
    from paper_2410_12707_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    B.load_library()  # fails loudly when the HIP library is not built

    w = {"1": wl.config1, "2a": lambda: wl.config2((1, 1000)), "2": lambda: wl.config2((1, 100)),
         "2c": lambda: wl.config2((1, 10)), "3": wl.config3, "4": wl.config4, "5": wl.config5,
         "5h": wl.config5_f16, "small": wl.config_small, "r18": wl.config_resnet18_samples}[args.config]()
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[w.dtype]
    esize = 4 if w.dtype == "f32" else 2
    graph_timed = args.config in ("small", "r18")
    S = len(w.tensors)
    n = w.n_total
    ks = list(w.ks)
    k = sum(ks)
    off = [0]
    for v in ks:
        off.append(off[-1] + v)

    def upload(t):
        if w.dtype == "bf16":
            return torch.from_numpy(t.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(t).cuda()

    # distinct input copies so that no step finds its input in the 256 MB last-level cache
    NBUF = 4 if S == 1 else 1  # the segmented batch (805 MB) is larger than that cache by itself
    xs = [[upload(t) for t in w.tensors] for _ in range(NBUF)]
    x_host = w.tensors[0]
    idx = torch.empty(max(k, 1), dtype=torch.int32, device="cuda")
    val = torch.empty(max(k, 1), dtype=tdt, device="cuda")
    err = torch.empty(S, dtype=torch.float32, device="cuda")
    ys = [torch.empty(t.size, dtype=tdt, device="cuda") for t in w.tensors]
    y = ys[0]
    ws = B.new_workspace(n, S, tdt)

    def step(i: int) -> None:
        if S == 1:
            B.adatopk_compress(xs[i % NBUF][0], k, idx, val, err, ws)
            B.adatopk_decompress_sorted(idx, val, k, y)
        else:
            B.adatopk_compress_segmented(xs[i % NBUF], ks, idx, val, off, err, ws)
            B.adatopk_decompress_segmented(idx, val, off, ys)

    run_step = step
    if graph_timed:  # one step captured once and replayed: no per-step marshalling on the host
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            step(0)
            side.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                step(0)
        torch.cuda.synchronize()

        def run_step(i: int) -> None:
            graph.replay()

    for i in range(args.warmup):
        run_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run_step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec_per_step = (t1 - t0) / args.steps
    dense_bytes = n * esize
    value = dense_bytes / sec_per_step / 1e9

    if args.calibrate_copy:
        for i in range(max(args.steps, 3)):
            B.measure_copy(y, xs[i % NBUF][0])  # reads and writes the bytes of one tensor
        torch.cuda.synchronize()

    # same loop on one buffer only (input may be served by the last-level cache): reported aside
    for i in range(args.warmup):
        run_step(0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run_step(0)
    torch.cuda.synchronize()
    warm_sec = (time.perf_counter() - t0) / args.steps

    # per-kernel durations: HIP events recorded by the library on the launch stream, same rotation
    names = B.measure_stage_names()
    B.measure_enable(True)
    acc = [0.0] * len(names)
    cnt = [0] * len(names)
    for i in range(args.steps):
        step(i)
        for j, ms in enumerate(B.measure_read()):
            if ms >= 0:
                acc[j] += ms
                cnt[j] += 1
    B.measure_enable(False)
    stage_us = {nm: (1e3 * acc[j] / cnt[j] if cnt[j] else None) for j, nm in enumerate(names)}

    # the two calls of a step timed apart
    def compress_only(i: int) -> None:
        if S == 1:
            B.adatopk_compress(xs[i % NBUF][0], k, idx, val, err, ws)
        else:
            B.adatopk_compress_segmented(xs[i % NBUF], ks, idx, val, off, err, ws)

    def decompress_only(i: int) -> None:
        if S == 1:
            B.adatopk_decompress_sorted(idx, val, k, y)
        else:
            B.adatopk_decompress_segmented(idx, val, off, ys)

    times = call_times(B, torch, compress_only, decompress_only, max(args.steps, 50)) if not graph_timed else {}

    # algorithmic bytes per launch of the full-size kernels (b bytes per value, n elements, k kept);
    # the segmented workload decompresses all its tensors in one k_merge launch as well
    b = esize
    algo = {
        "k_hist1": b * n,                          # one read of the input
        "k_gather": b * n + (4 + b) * k,           # second read of the input + the (index, value) pairs
        "k_merge": b * n + (4 + b) * k,            # one write of the dense output + the pairs read
        "k_small": b * n + (4 + b) * k,            # one-launch path: one read of the input + the pairs
    }
    algo = {nm: v for nm, v in algo.items() if stage_us.get(nm) is not None}
    dom = max(algo, key=lambda nm: stage_us[nm] or 0.0)
    dom_s = stage_us[dom] * 1e-6
    achieved = algo[dom] / dom_s / 1e9
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": TRAFFIC_BYTES.get(dom) if args.config == "2" else None,
                "algorithmic_bytes": algo[dom], "avg_us": round(stage_us[dom], 2)}

    # bytes the whole step must move (12 B/element + the pairs written and read back) against peak
    step_bytes = 3 * b * n + 2 * (4 + b) * k
    out = {
        "metric": "compress+decompress dense-input GB/s (fraction of HBM peak) at k=1%",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u32" if w.dtype == "f32" else "u16", "data": "synthetic",
        "config": {"workload": "%s: %s, %d tensor(s), n=%d, k=%d" % (w.name, w.note, S, n, k),
                   "input_rotation": "%d distinct input buffers (%d MB)" % (NBUF, NBUF * dense_bytes // 10**6),
                   "timed_as": "HIP graph replay of one step" if graph_timed else "eager calls"},
        "elements_per_s": round(n / sec_per_step, 0),
        "hbm_fraction_of_peak_min_traffic": round(step_bytes / sec_per_step / 1e9 / HBM_PEAK_GBS, 4),
        # the same with the bytes the counters saw for the five kernels of a step (headline workload only)
        "hbm_fraction_of_peak_measured_traffic": (round(sum(TRAFFIC_BYTES.values()) / sec_per_step / 1e9 / HBM_PEAK_GBS, 4)
                                                  if args.config == "2" else None),
        "warm_single_buffer": {"value": round(dense_bytes / warm_sec / 1e9, 1), "ms_per_step": round(warm_sec * 1e3, 5)},
        "stage_us": {nm: (round(v, 2) if v is not None else None) for nm, v in stage_us.items()},
        "roofline": roofline,
    }
    out.update(times)

    if S == 1 and not args.no_extras:
        out["micro_batch_pipeline"] = micro_batch_pipeline(B, torch, xs, k, tdt, n, esize, ws)
        out["concurrent_streams"] = concurrent_streams(B, torch, xs, k, tdt, n, esize)
        whole16 = (n * esize // 16) * 16 // esize
        out["streaming_ceiling"] = streaming_ceilings(B, torch, xs[0][0][:whole16], y[:whole16])

    if not args.no_cpu_baseline:
        from oracle import adatopk_oracle as orc

        # the oracle as it stands, single thread, on the first tensor of the workload (all of it when S = 1)
        step(0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ri, rv, re = orc.compress(x_host, ks[0])
        ry = orc.decompress(ri, rv, x_host.size)
        cpu_sec = time.perf_counter() - t0
        def to_np(t):
            t = t.cpu()
            return t.view(torch.int16).numpy().view(np.uint16) if w.dtype == "bf16" else t.numpy()

        gi = idx[:ks[0]].cpu().numpy()
        gv = to_np(val[:ks[0]])
        gy = to_np(ys[0])
        bits = (lambda a_: a_.view(np.uint32)) if w.dtype == "f32" else (lambda a_: a_.view(np.uint16))
        ok = (np.array_equal(gi, ri) and np.array_equal(bits(gv), bits(rv)) and np.array_equal(bits(gy), bits(ry))
              and abs(float(err.cpu()[0]) - float(re)) <= 1e-5 * float(re))
        out["cpu_baseline"] = {"value": round(x_host.size * esize / cpu_sec / 1e9, 5), "unit": "GB/s", "cores": 1,
                               "kind": "oracle", "seconds": round(cpu_sec, 3),
                               "sample": "tensor 1 of %d of the workload, whole (1 compress + 1 decompress of %d elements)"
                                         % (S, x_host.size)}
        out["parity_with_oracle"] = bool(ok)
        if S > 1:
            # the same oracle over every tensor of the batch, one host thread per tensor up to the
            # GPU machine's share of cores (the oracle's C code runs outside the interpreter lock)
            from concurrent.futures import ThreadPoolExecutor

            cores = min(S, 16, os.cpu_count() or 1)

            def one(s_):
                ri_, rv_, _ = orc.compress(w.tensors[s_], ks[s_])
                orc.decompress(ri_, rv_, w.tensors[s_].size)

            t0 = time.perf_counter()
            with ThreadPoolExecutor(max_workers=cores) as pool:
                list(pool.map(one, range(S)))
            par_sec = time.perf_counter() - t0
            out["cpu_baseline_all_tensors"] = {"value": round(n * esize / par_sec / 1e9, 5), "unit": "GB/s", "cores": cores,
                                               "host_threads_total": os.cpu_count(), "kind": "oracle",
                                               "seconds": round(par_sec, 3),
                                               "sample": "all %d tensors of the workload, one thread per tensor" % S}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
