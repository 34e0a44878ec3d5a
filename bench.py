#!/usr/bin/env python3
"""Benchmark of the AdaTopK hot path on one MI355X.

A step is one pass of the whole path over one tensor: adatopk_compress (threshold select,
stable compaction, error norm) followed by adatopk_decompress_sorted (zero fill + scatter of the
ascending pairs that compress wrote, one kernel), through the C ABI, on the GPT-2-small post-GELU
activation fp32 [32,1024,768] at k = 1 %.  Inputs are resident in HBM before the timed region; the
timed steps rotate over four distinct copies of the input (403 MB, more than the 256 MB last-level
cache) so that no step finds its input cached from the step before.  Prints ONE JSON line.

`value` comes from the wall clock around exactly --steps steps.  Everything that describes the
kernels (the step's median, the per-kernel durations, the roofline) is the median over at least
100 event-timed launches whatever --steps is, so that one slow launch does not move it.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak
MIN_TIMED = 100        # launches behind every median
KERNEL_SOURCE = os.path.join(ROOT, "paper_2410_12707_amd", "csrc", "adatopk.hip")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_cfg2_k1pct.json")

WORKLOADS = ["1", "2a", "2", "2c", "3", "4", "4r", "5", "5h", "small", "r18"]


def kernel_source_sha() -> str:
    with open(KERNEL_SOURCE, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()


def measured_traffic():
    """HBM bytes per launch from the counter runs (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by the
    plain copy kernel), as `bench.py --write-traffic` stored them together with the hash of the kernel
    source they were measured on.  None when the kernels have changed since: a stale figure is no figure."""
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return None
    return t if t.get("kernel_source_sha256") == kernel_source_sha() else None


def write_traffic(fetch_db: str, write_db: str, copy_bytes: int) -> int:
    """Turns the two counter runs of the headline workload (results databases of rocprofv3 --pmc FETCH_SIZE
    and --pmc WRITE_SIZE over `bench.py --calibrate-copy`) into profiles/hbm_traffic_cfg2_k1pct.json."""
    import sqlite3

    def per_kernel(db):
        con = sqlite3.connect(db)
        tables = [r[0] for r in con.execute("select name from sqlite_master where type in ('table','view')")]
        view = "counters_collection" if "counters_collection" in tables else None
        if view is None:
            raise SystemExit("no counters_collection view in %s" % db)
        out = {}
        for name, value, count in con.execute(
                "select kernel_name, avg(value), count(*) from %s group by kernel_name" % view):
            full = name.replace("(anonymous namespace)::", "").replace("void ", "").split("(")[0]
            short = full.split("<")[0]
            if short == "k_scan" and "true" in full:  # k_scan<dtype, speculative, depth>: the measuring build's stage names
                short = "k_scan_spec"
            out[short] = (float(value), int(count))
        return out

    f, w = per_kernel(fetch_db), per_kernel(write_db)
    if "k_copy16" not in f or "k_copy16" not in w:
        raise SystemExit("the counter runs must include the calibration copy (bench.py --calibrate-copy)")
    f_scale = copy_bytes / 1024.0 / f["k_copy16"][0]
    w_scale = copy_bytes / 1024.0 / w["k_copy16"][0]
    kernels = {}
    for name in sorted(f):
        if name == "k_copy16" or name not in w or not name.startswith("k_"):
            continue
        kernels[name] = {"fetch_bytes": round(f[name][0] * f_scale * 1024), "write_bytes": round(w[name][0] * w_scale * 1024),
                         "dispatches": f[name][1]}
    doc = {"kernel_source_sha256": kernel_source_sha(), "workload": "config 2 at k = 1 %",
           "unit": "bytes per dispatch, average over the run's dispatches",
           "calibration": {"copy_bytes": copy_bytes, "fetch_size_kib_reported": f["k_copy16"][0],
                           "write_size_kib_reported": w["k_copy16"][0], "fetch_scale": f_scale, "write_scale": w_scale},
           "kernels": kernels}
    with open(TRAFFIC_FILE, "w") as out:
        json.dump(doc, out, indent=1, sort_keys=True)
        out.write("\n")
    print("wrote %s (%d kernels)" % (TRAFFIC_FILE, len(kernels)))
    return 0


def median(v):
    s = sorted(v)
    return s[len(s) // 2]


def load_workload(wl, name):
    return {"1": wl.config1, "2a": lambda: wl.config2((1, 1000)), "2": lambda: wl.config2((1, 100)),
            "2c": lambda: wl.config2((1, 10)), "3": wl.config3, "4": wl.config4, "4r": wl.config4_links, "5": wl.config5,
            "5h": wl.config5_f16, "small": wl.config_small, "r18": wl.config_resnet18_samples}[name]()


class Bench:
    """One workload resident on the GPU with everything a step needs."""

    def __init__(self, B, torch, np, w, graph_timed: bool):
        self.B, self.torch, self.np, self.w = B, torch, np, w
        self.tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[w.dtype]
        self.esize = 4 if w.dtype == "f32" else 2
        self.S = len(w.tensors)
        self.n = w.n_total
        self.ratios = None
        if not w.ks:  # keep counts planned by the library from the workload's link parameters (Sec. 3.5, Eq. "adacompress")
            self.ratios, w.ks = B.adatopk_plan_keep_counts(w.alpha, w.beta, [t.size for t in w.tensors],
                                                           B._dtype_code(self.tdt), w.r_user, w.coeff)
        self.ks = list(w.ks)
        self.k = sum(self.ks)
        self.off = [0]
        for v in self.ks:
            self.off.append(self.off[-1] + v)
        # distinct input copies so that no step finds its input in the 256 MB last-level cache
        self.NBUF = 4 if self.S == 1 else 1  # a batch of tensors is larger than that cache by itself or launch-bound
        self.xs = [[self.upload(t) for t in w.tensors] for _ in range(self.NBUF)]
        self.idx = torch.empty(max(self.k, 1), dtype=torch.int32, device="cuda")
        self.val = torch.empty(max(self.k, 1), dtype=self.tdt, device="cuda")
        self.err = torch.empty(self.S, dtype=torch.float32, device="cuda")
        self.ys = [torch.empty(t.size, dtype=self.tdt, device="cuda") for t in w.tensors]
        self.ws = B.new_workspace(self.n, self.S, self.tdt)
        self.graph = None
        if graph_timed:  # one step captured once and replayed: no per-step marshalling on the host
            side = torch.cuda.Stream()
            with torch.cuda.stream(side):
                self.step(0)
                side.synchronize()
                self.graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(self.graph, stream=side):
                    self.step(0)
            torch.cuda.synchronize()

    def upload(self, t):
        if self.w.dtype == "bf16":
            return self.torch.from_numpy(t.view(self.np.int16)).cuda().view(self.torch.bfloat16)
        return self.torch.from_numpy(t).cuda()

    def compress(self, i: int) -> None:
        B = self.B
        if self.S == 1:
            B.adatopk_compress(self.xs[i % self.NBUF][0], self.k, self.idx, self.val, self.err, self.ws)
        else:
            B.adatopk_compress_segmented(self.xs[i % self.NBUF], self.ks, self.idx, self.val, self.off, self.err, self.ws)

    def decompress(self, i: int) -> None:
        B = self.B
        if self.S == 1:
            B.adatopk_decompress_sorted(self.idx, self.val, self.k, self.ys[0])
        else:
            B.adatopk_decompress_segmented(self.idx, self.val, self.off, self.ys)

    def step(self, i: int) -> None:
        self.compress(i)
        self.decompress(i)

    def run(self, i: int) -> None:
        if self.graph is not None:
            self.graph.replay()
        else:
            self.step(i)

    def wall_clock(self, steps: int, warmup: int, rotate: bool = True) -> float:
        """Seconds per step: exactly `steps` steps between two synchronisations, after `warmup` untimed ones."""
        torch = self.torch
        for i in range(warmup):
            self.run(i if rotate else 0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.run(i if rotate else 0)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def event_timed(self, fn, reps: int):
        """Microseconds of `reps` calls of fn(i), each between an event pair of its own on the launch stream."""
        torch = self.torch
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        torch.cuda.synchronize()
        for i, (e0, e1) in enumerate(evs):
            e0.record()
            fn(i)
            e1.record()
        torch.cuda.synchronize()
        return [e0.elapsed_time(e1) * 1e3 for e0, e1 in evs]

    def stage_medians(self, reps: int):
        """Median duration in microseconds of every kernel of a step, from the measuring build of the library
        (the same sources; every launch carries start / stop events with the dispatch's own timestamps,
        which is what rocprofv3 --kernel-trace reports as well), over `reps` steps with rotating inputs."""
        B = self.B
        names = B.measure_stage_names()
        seen = [[] for _ in names]
        with B.measuring():
            for i in range(3):
                self.step(i)
            self.torch.cuda.synchronize()
            B.measure_read()
            for i in range(reps):
                self.step(i)
                for j, ms in enumerate(B.measure_read()):
                    if ms >= 0:
                        seen[j].append(ms * 1e3)
        return {nm: {"median_us": round(median(v), 2), "min_us": round(min(v), 2), "max_us": round(max(v), 2),
                     "launches": len(v)} for nm, v in zip(names, seen) if v}

    def algorithmic_bytes(self):
        """What each full-size kernel must move per launch (b bytes per value, n elements, k kept)."""
        b, n, k = self.esize, self.n, self.k
        return {
            "k_scan_spec": b * n + (4 + b) * k,  # one read of the input + the candidate pairs written (at least the k kept ones)
            "k_hist1": b * n,                    # exact passes (when they do not return at once): one read of the input ...
            "k_scan": b * n + (4 + b) * k,       # ... and another, with the candidate pairs written
            "k_merge": b * n + (4 + b) * k,      # one write of the dense output + the pairs read
            "k_small": b * n + (4 + b) * k,      # one-launch path: one read of the input + the pairs
        }

    def step_bytes(self, input_reads: int) -> int:
        """Bytes a step moves at the least: `input_reads` full reads of the input (one when the speculative
        pass holds, two for the exact passes), the output written once, the kept pairs written and read back."""
        return (input_reads + 1) * self.esize * self.n + 2 * (4 + self.esize) * self.k

    def parity(self, orc, s: int = 0) -> bool:
        """Tensor s of the workload, whole, against the oracle: indices, values, reconstruction, error norm."""
        np, torch, w = self.np, self.torch, self.w
        self.step(0)
        torch.cuda.synchronize()
        x = w.tensors[s]
        ri, rv, re = orc.compress(x, self.ks[s])
        ry = orc.decompress(ri, rv, x.size)

        def to_np(t):
            t = t.cpu()
            return t.view(torch.int16).numpy().view(np.uint16) if w.dtype == "bf16" else t.numpy()

        bits = (lambda a_: a_.view(np.uint32)) if w.dtype == "f32" else (lambda a_: a_.view(np.uint16))
        gi = self.idx[self.off[s]:self.off[s + 1]].cpu().numpy()
        gv = to_np(self.val[self.off[s]:self.off[s + 1]])
        gy = to_np(self.ys[s])
        ge = float(self.err.cpu()[s])
        return bool(np.array_equal(gi, ri) and np.array_equal(bits(gv), bits(rv)) and np.array_equal(bits(gy), bits(ry))
                    and abs(ge - float(re)) <= 1e-5 * float(re))


def micro_batch_pipeline(bench, n_b=4, rounds=25, pair_matrix=False):
    """Sender side of pipeline parallelism with n_b micro-batches (paper Sec. 3.6): every micro-batch's
    activation is compressed straight into a wire message, and the message is copied to pinned host
    memory, where a network stack would pick it up.  Serial: both on one stream.  Overlapped: the copy
    of micro-batch j runs on a second stream while the next micro-batches are compressed (n_b message buffers).

    In the overlapped form the host waits for a message buffer's copy before it enqueues the compress that
    fills the buffer again, so it is never more than n_b micro-batches ahead of the GPU (a sender with n_b
    buffers has to; run far ahead, the enqueue calls themselves were seen to get 2.3 times slower for whole runs).
    The overlapped form is bound by the host, not by the GPU: one micro-batch costs the host six kernel
    launches, two event records, two cross-stream waits and one asynchronous copy, 60 to 73 us of enqueue
    time against about 50 us of GPU time per micro-batch, so the time the host spends in the loop is
    reported beside the total.  On top of that the stream pair matters: HIP spreads its streams over a few
    hardware queues (four on this machine) and some pairs run 2.5 to 3.5 times slower than the rest, for
    as long as the process lives.  Nothing in the API tells such a pair apart, so the copy stream is chosen
    the way an executor has to choose it: by timing a short run with each of a handful of candidates.
    Returns microseconds per micro-batch; with pair_matrix the overlapped time of every pair of eight
    streams as well."""
    B, torch, xs, k, n, ws = bench.B, bench.torch, bench.xs, bench.k, bench.n, bench.ws
    dt_code = B._dtype_code(bench.tdt)
    nbytes = B.adatopk_wire_bytes(k, dt_code, 4)
    nbuf = n_b  # one message buffer per micro-batch in flight: a buffer is waited for only every n_b-th time
    wire = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(nbuf)]
    host = [torch.empty(nbytes, dtype=torch.uint8, pin_memory=True) for _ in range(nbuf)]
    pool = [torch.cuda.Stream() for _ in range(8 if pair_matrix else 5)]
    comp = pool[0]
    done = [torch.cuda.Event() for _ in range(nbuf)]
    freed = [torch.cuda.Event() for _ in range(nbuf)]

    host_share = []  # per run: the part of its time the host spent enqueueing

    def run(copy, reps=rounds, comp=comp) -> float:  # copy is None: everything on the compress stream
        torch.cuda.synchronize()
        for e in freed:
            e.record(comp)
        t0 = time.perf_counter()
        for j in range(n_b * reps):
            b = j % nbuf
            if copy is not None and j >= nbuf:
                freed[b].synchronize()  # the sender owns n_b message buffers: it waits for one before it fills it again
            with torch.cuda.stream(comp):
                if copy is None or j < nbuf:
                    comp.wait_event(freed[b])
                B.adatopk_compress_wire(xs[j % len(xs)][0], k, 4, float(n) / max(k, 1), wire[b], ws)
                done[b].record(comp)
            with torch.cuda.stream(copy if copy is not None else comp):
                if copy is not None:
                    copy.wait_event(done[b])
                host[b].copy_(wire[b], non_blocking=True)
                freed[b].record(copy if copy is not None else comp)
        t1 = time.perf_counter()
        torch.cuda.synchronize()
        host_share.append((t1 - t0) / (n_b * reps) * 1e6)
        return (time.perf_counter() - t0) / (n_b * reps) * 1e6

    def run_zero_copy() -> float:  # the kernels write the message straight into pinned host memory
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(comp):
            for j in range(n_b * rounds):
                B.adatopk_compress_wire(xs[j % len(xs)][0], k, 4, float(n) / max(k, 1), host[j % nbuf], ws)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / (n_b * rounds) * 1e6

    run(pool[1])  # warm-up of all paths
    run_zero_copy()
    zero_copy = sorted(run_zero_copy() for _ in range(5))
    serial = sorted(run(None) for _ in range(5))
    probe = [min(run(c, reps=5) for _ in range(2)) for c in pool[1:5]]  # the executor's choice of a copy stream
    chosen = pool[1 + probe.index(min(probe))]
    del host_share[:]
    overlapped = sorted(run(chosen) for _ in range(5))
    enqueue = sorted(host_share)[2]
    out = {"n_b": n_b, "message_bytes": nbytes, "serial_us_per_micro_batch": round(serial[2], 2),
           "overlapped_us_per_micro_batch": round(overlapped[2], 2),
           "overlapped_us_runs": [round(v, 1) for v in overlapped],
           "overlapped_host_enqueue_us_per_micro_batch": round(enqueue, 2),
           "copy_stream_candidates_us": [round(v, 1) for v in probe],
           "into_pinned_host_us_per_micro_batch": round(zero_copy[2], 2),
           "what": "compress into a wire message + copy of the message to pinned host memory (serial: one stream; "
                   "overlapped: copies on a second stream, the fastest of four candidates in a short trial, since some "
                   "stream pairs are several times slower than others; the host's enqueue time per micro-batch is given "
                   "because it, not the GPU, bounds the overlapped form), or the message written "
                   "by the kernels straight into pinned host memory; median of 5 runs of %d micro-batches" % (n_b * rounds)}
    if pair_matrix:
        out["overlapped_us_by_stream_pair"] = [[None if i == j else round(sorted(run(pool[j], reps=10, comp=pool[i])
                                                                                 for _ in range(3))[1], 1)
                                                for j in range(8)] for i in range(8)]
    return out


def concurrent_streams(bench, streams=4, rounds=50):
    """Independent compress + decompress steps on several streams, each with its own workspace and
    outputs: what the GPU sustains when the tensors of several pipeline edges are in flight at once."""
    B, torch, xs, k, n, tdt = bench.B, bench.torch, bench.xs, bench.k, bench.n, bench.tdt
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
    return {"streams": streams, "us_per_step": round(sec * 1e6, 2), "value": round(n * bench.esize / sec / 1e9, 1), "unit": "GB/s"}


def streaming_ceilings(bench, reps=50):
    """What the memory system gives plain kernels (of the library's measuring build) on a buffer of the
    tensor's size: read only, fill only, copy (GB/s of bytes moved; the copy moves twice the buffer)."""
    B, torch = bench.B, bench.torch
    whole16 = (bench.n * bench.esize // 16) * 16 // bench.esize
    src, dst = bench.xs[0][0][:whole16], bench.ys[0][:whole16]
    nbytes = src.numel() * src.element_size()
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = {}
    for name, fn, moved in (("read", lambda i: B.measure_read_only(src, sink), nbytes),
                            ("fill", lambda i: B.measure_fill(dst), nbytes),
                            ("copy", lambda i: B.measure_copy(dst, src), 2 * nbytes)):
        fn(0)
        out[name] = round(moved / (median(bench.event_timed(fn, reps)) * 1e-6) / 1e9, 1)
    out["unit"] = "GB/s"
    out["bytes"] = nbytes
    return out


def other_config_line(B, torch, np, wl, orc, name):
    """Step time of one of the other parity configurations, event-timed, with its fractions of peak."""
    w = load_workload(wl, name)
    bench = Bench(B, torch, np, w, graph_timed=False)
    for i in range(10):
        bench.step(i)
    us = bench.event_timed(bench.step, MIN_TIMED)
    med = median(us)
    dense = bench.n * bench.esize
    stage_us = {nm: v["median_us"] for nm, v in bench.stage_medians(20).items()}
    reads = sum(1 for nm in ("k_scan_spec", "k_hist1", "k_scan", "k_small")
                if nm in stage_us and bench.esize * bench.n / stage_us[nm] / 1e3 <= HBM_PEAK_GBS)
    line = {"config": name, "workload": w.name, "dtype": w.dtype, "tensors": bench.S, "n": bench.n, "k": bench.k,
            "step_us_median": round(med, 2), "step_us_min_max": [round(min(us), 2), round(max(us), 2)],
            "dense_input_GBs": round(dense / med / 1e3, 1), "stage_us": stage_us, "input_reads_per_step": reads,
            "hbm_fraction_of_peak_min_traffic": round(bench.step_bytes(reads) / med / 1e3 / HBM_PEAK_GBS, 4)}
    if orc is not None and name in ("1", "5"):
        line["parity_with_oracle"] = bench.parity(orc)
    del bench
    torch.cuda.empty_cache()
    return line


def value_structures(B, torch, np, wl, n=32 * 1024 * 768, reps=30):
    """Compress + decompress of one fp32 tensor of config 2's size at k = 1 % for value structures that a
    radix select or a compaction can be slow on (constant, all zero, sorted, few distinct values, one narrow
    bucket, mostly zeros) beside the two benign ones.  Per structure: the median step (event pairs), whether the
    sample-based window held, and the median duration of every kernel (measuring build)."""
    k = n // 100
    rng = np.random.Generator(np.random.PCG64(5))
    kinds = {"normal": lambda: rng.standard_normal(n, dtype=np.float32),
             "uniform": lambda: rng.random(n, dtype=np.float32),
             "few_levels": lambda: wl.small_case("few_levels", n, 3),
             "mostly_zero_97pct": lambda: wl.small_case("sparse", n, 3),
             "ascending": lambda: np.arange(1, n + 1, dtype=np.float64).astype(np.float32),
             "descending": lambda: np.arange(n, 0, -1, dtype=np.float64).astype(np.float32),  # (in fp32 the step rounds to 0 above 2^24)
             "one_bucket": lambda: (1.0 + rng.random(n, dtype=np.float32) * 0.08).astype(np.float32),
             "all_equal": lambda: np.full(n, 1.5, dtype=np.float32),
             "all_zero": lambda: np.zeros(n, dtype=np.float32)}
    idx = torch.empty(k, dtype=torch.int32, device="cuda")
    val = torch.empty(k, device="cuda")
    err = torch.empty(1, device="cuda")
    y = torch.empty(n, device="cuda")
    ws = B.new_workspace(n, 1, torch.float32)
    out = []
    for kind, make in kinds.items():
        x = torch.from_numpy(make()).cuda()

        def step():
            B.adatopk_compress(x, k, idx, val, err, ws)
            B.adatopk_decompress_sorted(idx, val, k, y)

        for _ in range(5):
            step()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        torch.cuda.synchronize()
        for a, b in evs:
            a.record()
            step()
            b.record()
        torch.cuda.synchronize()
        us = median([a.elapsed_time(b) * 1e3 for a, b in evs])
        held = int(ws[:64].view(torch.int32)[6].item())  # the tensor's state record: did the sample-based window hold
        seen = {}
        with B.measuring():
            for _ in range(10):
                step()
                for name, ms in zip(B.measure_stage_names(), B.measure_read()):
                    if ms >= 0:
                        seen.setdefault(name, []).append(ms * 1e3)
        out.append({"values": kind, "step_us_median": round(us, 1), "sample_window_held": bool(held),
                    "stage_us": {name: round(median(v), 1) for name, v in seen.items()}})
        del x
    return {"n": n, "k": k, "dtype": "f32", "structures": out}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--config", default="2", choices=WORKLOADS,
                    help="workload: 2 (default, the headline: GELU tensor at k = 1 %%), 2a / 2c = the same tensor at "
                         "k = 0.1 %% / 10 %%, 1, 3, 4 (segmented batch), 5 (bf16) = the other parity configurations; "
                         "4r = config 4's tensors with the keep counts planned by the library from 8 Mbps - 10 Gbps "
                         "link parameters (the bandwidth-adaptive rule end to end); 5h = config 5 in fp16; small = 128 "
                         "messages of 1024-8192 elements in one call, r18 = 64 per-sample ResNet-18 stage outputs in "
                         "one call (both timed as HIP graph replays: the Python marshalling of that many pointers "
                         "would otherwise be the bottleneck)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the side measurements (micro-batch pipeline, concurrent streams, the other configurations)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run the plain copy kernel on the workload-sized buffer (the known-size kernel that "
                         "hardware-counter readings are scaled by)")
    ap.add_argument("--stream-pairs", action="store_true",
                    help="no benchmark line: time the micro-batch pipeline (compress on one stream, message copies on "
                         "another) for every pair of eight streams and print the matrix")
    ap.add_argument("--value-structures", action="store_true",
                    help="no benchmark line: compress + decompress of a 25 M-element fp32 tensor at k = 1 %% for constant, "
                         "zero, sorted, few-valued, narrow-range and mostly-zero tensors, with the kernels' durations")
    ap.add_argument("--min-timed", type=int, default=MIN_TIMED,
                    help="launches behind every median (default %d; hardware-counter runs, where every dispatch is "
                         "slow and only the counters matter, use fewer)" % MIN_TIMED)
    ap.add_argument("--write-traffic", nargs=2, metavar=("FETCH_DB", "WRITE_DB"),
                    help="no benchmark: read the results databases of two counter runs of the default workload "
                         "(rocprofv3 --pmc FETCH_SIZE / --pmc WRITE_SIZE -- python3 bench.py --calibrate-copy ...) and "
                         "store the bytes per kernel launch, with the hash of the kernel source, under profiles/")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2
    if args.write_traffic:
        return write_traffic(args.write_traffic[0], args.write_traffic[1], 32 * 1024 * 768 * 4)

    import numpy as np
    import torch

    from paper_2410_12707_amd import binding as B
    from paper_2410_12707_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    B.load_library()  # fails loudly when the HIP library is not built

    if args.value_structures:
        r = value_structures(B, torch, np, wl)
        print(json.dumps(r))
        for row in r["structures"]:
            print("%-18s %7.1f us  window held: %-5s %s" % (row["values"], row["step_us_median"], row["sample_window_held"],
                                                          "  ".join("%s %.1f" % kv for kv in row["stage_us"].items())))
        return 0
    w = load_workload(wl, args.config)
    graph_timed = args.config in ("small", "r18")
    bench = Bench(B, torch, np, w, graph_timed)
    S, n, k, esize = bench.S, bench.n, bench.k, bench.esize
    dense_bytes = n * esize
    reps = max(args.steps, args.min_timed)
    if args.stream_pairs:
        r = micro_batch_pipeline(bench, pair_matrix=True)
        print(json.dumps({k_: v for k_, v in r.items() if k_ != "what"}))
        print("overlapped us per micro-batch; row = compress stream, column = copy stream (streams in creation order)")
        for row in r["overlapped_us_by_stream_pair"]:
            print(" ".join("   -  " if v is None else "%6.1f" % v for v in row))
        return 0

    # the contract's number: wall clock around exactly --steps steps, inputs rotating
    sec_per_step = bench.wall_clock(args.steps, args.warmup)
    value = dense_bytes / sec_per_step / 1e9

    if args.calibrate_copy:
        for i in range(max(args.steps, 3)):
            B.measure_copy(bench.ys[0], bench.xs[i % bench.NBUF][0])  # reads and writes the bytes of one tensor
        torch.cuda.synchronize()

    # the same step between event pairs: median and spread over at least MIN_TIMED launches
    step_us = bench.event_timed(bench.run, reps)
    # one buffer only (the input may then be served by the last-level cache): reported aside
    warm_us = bench.event_timed(lambda i: bench.run(0), reps)
    stages = bench.stage_medians(reps)
    stage_us = {nm: v["median_us"] for nm, v in stages.items()}

    # the two calls of a step timed apart
    times = {}
    if not graph_timed:
        times = {"t_compress_us": round(median(bench.event_timed(bench.compress, reps)), 2),
                 "t_decompress_us": round(median(bench.event_timed(bench.decompress, reps)), 2)}

    # roofline of the full-size kernels: algorithmic bytes per launch over the median launch duration.  A
    # pass over the input that finishes faster than the peak allows did not read it: the exact passes
    # return at once when the speculative pass held (and the other way round), so they are left out.
    algo = {nm: v for nm, v in bench.algorithmic_bytes().items()
            if nm in stage_us and v / stage_us[nm] / 1e3 <= HBM_PEAK_GBS}
    input_reads = sum(1 for nm in ("k_scan_spec", "k_hist1", "k_scan", "k_small") if nm in algo)
    traffic = measured_traffic() if args.config == "2" else None

    def roof(nm):
        achieved = algo[nm] / stage_us[nm] / 1e3
        t = traffic["kernels"].get(nm) if traffic else None
        return {"bound": "hbm", "kernel": nm, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": (t["fetch_bytes"] + t["write_bytes"]) if t else None,
                "algorithmic_bytes": algo[nm], "median_us": stage_us[nm],
                "min_max_us": [stages[nm]["min_us"], stages[nm]["max_us"]], "launches": stages[nm]["launches"]}

    full = sorted(algo, key=lambda nm: -stage_us[nm])
    roofline = roof(full[0])  # the slowest full-size kernel
    roofline["traffic_source"] = ("profiles/%s (counter runs on this kernel source)" % os.path.basename(TRAFFIC_FILE)
                                  if traffic else "none for this kernel source / workload: not measured by this run")

    med = median(step_us)
    out = {
        "metric": "compress+decompress dense-input GB/s (fraction of HBM peak) at k=1%",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "%s: %s, %d tensor(s), n=%d, k=%d" % (w.name, w.note, S, n, k),
                   "input_rotation": "%d distinct input buffers (%d MB)" % (bench.NBUF, bench.NBUF * dense_bytes // 10**6),
                   "timed_as": "HIP graph replay of one step" if graph_timed else "eager calls"},
        "elements_per_s": round(n / sec_per_step, 0),
        "step_us_median": round(med, 2), "step_us_min_max": [round(min(step_us), 2), round(max(step_us), 2)],
        "step_launches_timed": len(step_us),
        "dense_input_GBs_at_median": round(dense_bytes / med / 1e3, 1),
        "input_reads_per_step": input_reads,
        "hbm_fraction_of_peak_min_traffic": round(bench.step_bytes(input_reads) / med / 1e3 / HBM_PEAK_GBS, 4),
        # the same with the bytes the counters saw for the kernels of a step (headline workload only)
        "hbm_fraction_of_peak_measured_traffic": (
            round(sum(t["fetch_bytes"] + t["write_bytes"] for t in traffic["kernels"].values()) / med / 1e3 / HBM_PEAK_GBS, 4)
            if traffic else None),
        "warm_single_buffer": {"step_us_median": round(median(warm_us), 2),
                               "value": round(dense_bytes / median(warm_us) / 1e3, 1)},
        "stage_us": stage_us,
        "roofline": roofline,
        "full_size_kernels": [roof(nm) for nm in full],
    }
    out.update(times)
    if bench.ratios is not None:
        out["planned_keep_counts"] = {"k": bench.ks, "ratio_min_max": [min(bench.ratios), max(bench.ratios)],
                                      "tensors_sent_uncompressed": sum(1 for k_, t in zip(bench.ks, w.tensors) if k_ == t.size)}

    orc = None
    if not args.no_cpu_baseline:
        from oracle import adatopk_oracle as orc

    if S == 1 and not args.no_extras:
        out["micro_batch_pipeline"] = micro_batch_pipeline(bench)
        out["concurrent_streams"] = concurrent_streams(bench)
        out["streaming_ceiling"] = streaming_ceilings(bench)

    if orc is not None:
        # the oracle as it stands, single thread, on the first tensor of the workload (all of it when S = 1)
        x_host = w.tensors[0]
        t0 = time.perf_counter()
        ri, rv, _ = orc.compress(x_host, bench.ks[0])
        orc.decompress(ri, rv, x_host.size)
        cpu_sec = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(x_host.size * esize / cpu_sec / 1e9, 5), "unit": "GB/s", "cores": 1,
                               "host_threads_total": os.cpu_count(), "kind": "oracle", "seconds": round(cpu_sec, 3),
                               "sample": "tensor 1 of %d of the workload, whole (1 compress + 1 decompress of %d elements)"
                                         % (S, x_host.size)}
        out["parity_with_oracle"] = bench.parity(orc)
        if S > 1:
            # the same oracle over every tensor of the batch, one host thread per tensor up to the
            # GPU machine's share of cores (the oracle's C code runs outside the interpreter lock)
            from concurrent.futures import ThreadPoolExecutor

            cores = min(S, 16, os.cpu_count() or 1)

            def one(s_):
                ri_, rv_, _ = orc.compress(w.tensors[s_], bench.ks[s_])
                orc.decompress(ri_, rv_, w.tensors[s_].size)

            t0 = time.perf_counter()
            with ThreadPoolExecutor(max_workers=cores) as pool:
                list(pool.map(one, range(S)))
            par_sec = time.perf_counter() - t0
            out["cpu_baseline_all_tensors"] = {"value": round(n * esize / par_sec / 1e9, 5), "unit": "GB/s", "cores": cores,
                                               "host_threads_total": os.cpu_count(), "kind": "oracle",
                                               "seconds": round(par_sec, 3),
                                               "sample": "all %d tensors of the workload, one thread per tensor" % S}

    if args.config == "2" and not args.no_extras:
        # the other parity configurations, event-timed by this same run (no CPU timing; parity for 1 and 5)
        del bench
        torch.cuda.empty_cache()
        out["other_configs"] = [other_config_line(B, torch, np, wl, orc, name) for name in ("1", "2a", "2c", "3", "4", "5")]
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
