"""Parity of the HIP path with the CPU oracle, element by element, through the C ABI.

Bar: indices, values and the reconstructed tensor bit-exact; the fp32 error norm within
1e-5 relative (the kernels accumulate in fp64 like the oracle, in another order).
"""
import numpy as np
import pytest

from oracle import adatopk_oracle as orc
from paper_2410_12707_amd import workloads as wl

pytestmark = pytest.mark.gpu

ERR_RTOL = 1e-5


def check_one(x, k, offset_elems=0, label=""):
    import gpu_harness as H

    n = x.size
    ri, rv, re = orc.compress(x, k)
    gi, gv, ge = H.gpu_compress(x, k, offset_elems)
    assert gi.size == k and np.array_equal(gi, ri), "indices differ " + label
    assert np.array_equal(H.bits(gv), H.bits(rv)), "values differ " + label
    assert H.same_err(ge, re, ERR_RTOL), "err %r vs %r %s" % (ge, re, label)
    ry = orc.decompress(ri, rv, n)
    gy = H.gpu_decompress(gi, gv, n, offset_elems)
    assert np.array_equal(H.bits(gy), H.bits(ry)), "reconstruction differs " + label
    gy = H.gpu_decompress(gi, gv, n, offset_elems, sorted_call=True)
    assert np.array_equal(H.bits(gy), H.bits(ry)), "reconstruction (ascending-index call) differs " + label


def ks_for(n):
    return sorted({0, 1, n // 100, n // 3, n - 1, n} & set(range(0, n + 1)))


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("kind", ["normal", "few_levels", "all_equal", "all_zero", "signed_zero_mix", "sparse",
                                  "nonfinite", "random_bits", "descending"])
def test_small_and_ragged_sizes(kind, dtype):
    # below one vector, one wavefront, one tile (8192 fp32 / 16384 bf16), a few tiles and a
    # ragged tail, several chunks
    for n in (1, 3, 64, 1000, 8192, 8193, 16385, 70001):
        x = wl.small_case(kind, n, seed=1000 + n, dtype=dtype)
        for k in ks_for(n):
            check_one(x, k, label="%s %s n=%d k=%d" % (kind, dtype, n, k))


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_many_chunks_and_tiles(dtype):
    # 3.3M elements: hundreds of chunks, several tiles each, ragged last chunk
    n = 3_300_017
    for kind, k in (("normal", n // 100), ("few_levels", n // 7), ("sparse", n // 20), ("random_bits", n // 1000)):
        check_one(wl.small_case(kind, n, seed=77, dtype=dtype), k, label="%s %s" % (kind, dtype))


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_misaligned_base_pointer(dtype):
    n = 40_003
    x = wl.small_case("normal", n, seed=5, dtype=dtype)
    for off in (1, 3):
        check_one(x, n // 50, offset_elems=off, label="offset %d" % off)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_dense_chunks_of_a_large_tensor_are_read_again_from_the_input(dtype):
    # One tensor of 11M elements: chunks of 40960+ elements, i.e. five and more tiles each.  Where more
    # than a quarter of a chunk are candidates its list overflows and the later kernels read the chunk
    # from the input again, tile after tile with loads in flight ahead (every branch of those loops
    # needs five tiles or more).  Constant tensor: every chunk, the quota of ties ends inside a tile.
    # Sorted: only the chunks at one end.  Clipped: ties at the largest value, spread over all chunks.
    n = 11_000_013
    rng = np.random.Generator(np.random.PCG64(17))
    clipped = np.clip(rng.standard_normal(n, dtype=np.float32), -0.5, 0.5)
    cases = [("all_equal", wl.small_case("all_equal", n, 3, dtype), n // 100 + 5),
             ("descending", wl.small_case("descending", n, 3, dtype), n // 100),
             ("ascending", wl.small_case("ascending", n, 3, dtype), n // 64 + 1),
             ("clipped", clipped if dtype == "f32" else (wl.f32_to_bf16_bits(clipped) if dtype == "bf16"
                                                         else clipped.astype(np.float16)), n // 50)]
    for name, x, k in cases:
        check_one(x, k, label="%s %s" % (name, dtype))
    # base pointer off the 16-byte grid: the counting kernel then takes the entry loop for the same chunks
    check_one(cases[0][1][: n // 2], n // 300, offset_elems=1, label="all_equal offset 1 %s" % dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chunks_kept_whole_in_a_batch_of_few_chunks(dtype):
    # Four tensors in one call, under 256 chunks of one tile together: the launch shape in which a batch
    # takes the list kernels' form for one workgroup per chunk, with dense chunks read in wide tiles.
    # Constant tensor (whole chunks kept, then the quota ends inside one), sorted either way (the last
    # chunk of the ascending one is short and kept whole), and an ordinary tensor between them.
    import gpu_harness as H

    ns = [500_000, 400_003, 300_000, 450_001]
    xs = [wl.small_case("all_equal", ns[0], 3, dtype), wl.small_case("descending", ns[1], 3, dtype),
          wl.small_case("normal", ns[2], 3, dtype), wl.small_case("ascending", ns[3], 3, dtype)]
    ks = [25_000 + 77, 40_000, 3_000, 8192 * 5 + 4321]
    gi, gv, off, ge = H.gpu_compress_segmented(xs, ks)
    for s, (x, k) in enumerate(zip(xs, ks)):
        ri, rv, re = orc.compress(x, k)
        assert np.array_equal(gi[off[s]:off[s + 1]], ri), "indices differ, tensor %d %s" % (s, dtype)
        assert np.array_equal(H.bits(gv[off[s]:off[s + 1]]), H.bits(rv)), "values differ, tensor %d %s" % (s, dtype)
        assert H.same_err(ge[s], re, ERR_RTOL), "err %r vs %r, tensor %d %s" % (ge[s], re, s, dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("share,width,kept", [(0.06, 200, range(60, 161, 10)), (0.03, 300, range(60, 221, 10)),
                                              (0.0046, 400, range(50, 301, 25))])
def test_error_norm_of_16bit_types_as_the_threshold_moves_through_the_window(dtype, share, width, kept):
    # A share of the elements is spread evenly over `width` consecutive 16-bit patterns, the rest lie far
    # below; k keeps a growing number of those patterns.  The window that the sample sets starts a certain
    # fraction of k below the threshold (the larger k, the smaller the fraction), so the three settings put
    # the threshold's window bin at 11-24, at 25-37 (29, 30, 31, 32, 33 among them) and at 90-145 (with the
    # thinnest spread the sample also misses at both ends of the range, and the exact passes run).  Up to
    # bin 30 the error norm takes the window's column sums from the bucket search, beyond it adds them up
    # itself.
    import gpu_harness as H

    n = (1 << 20) + 4099
    rng = np.random.Generator(np.random.PCG64(23))
    top = 0x4100 if dtype == "bf16" else 0x4A00  # patterns of 8.0 upwards (bf16) / 12.0 upwards (fp16)
    low = (0x3000, 0x3400) if dtype == "bf16" else (0x2000, 0x2800)
    pats = rng.integers(low[0], low[1], size=n, dtype=np.uint32).astype(np.uint16)
    spread = rng.random(n) < share
    pats[spread] = (top + rng.integers(0, width, size=int(spread.sum()))).astype(np.uint16)
    pats[rng.random(n) < 0.5] |= np.uint16(0x8000)
    x = pats if dtype == "bf16" else pats.view(np.float16)
    per_pattern = int(spread.sum()) // width
    for kept_patterns in kept:
        k = kept_patterns * per_pattern + 17
        ri, rv, re = orc.compress(x, k)
        gi, gv, ge = H.gpu_compress(x, k)
        assert np.array_equal(gi, ri) and np.array_equal(H.bits(gv), H.bits(rv)), (dtype, kept_patterns)
        assert H.same_err(ge, re, ERR_RTOL), "err %r vs %r with %d patterns kept, %s" % (ge, re, kept_patterns, dtype)


def test_ties_straddling_tiles_and_chunks():
    # the tied value sits on both sides of every tile and chunk boundary; the quota ends mid-way
    n = 300_000
    x = np.full(n, 0.5, dtype=np.float32)
    x[::3] = 2.0  # 100000 larger values
    x[1::8192] = -2.0
    for k in (1, 99_999, 100_000 + 37, 100_000 + 8192 * 5 + 1, n - 1):
        check_one(x, k, label="ties k=%d" % k)


def test_decompress_unsorted_and_out_of_range():
    import gpu_harness as H

    n = 100_000
    rng = np.random.Generator(np.random.PCG64(9))
    idx = rng.permutation(n)[:5000].astype(np.int32)
    val = rng.standard_normal(5000, dtype=np.float32)
    assert np.array_equal(H.bits(H.gpu_decompress(idx, val, n)), H.bits(orc.decompress(idx, val, n)))
    bad = idx.copy()
    bad[::10] = n + 5  # skipped by contract
    bad[1::10] = -3
    ok = (bad >= 0) & (bad < n)
    assert np.array_equal(H.bits(H.gpu_decompress(bad, val, n)), H.bits(orc.decompress(bad[ok], val[ok], n)))
    assert np.all(H.gpu_decompress(np.empty(0, np.int32), np.empty(0, np.float32), 1000) == 0)


def test_decompress_sorted_spans_and_misuse():
    import gpu_harness as H

    rng = np.random.Generator(np.random.PCG64(10))
    for n, k, dtype in ((5_000_011, 50_000, "f32"), (5_000_011, 50_000, "bf16"), (1_000_000, 1_000_000, "f32"),
                        (4097, 1, "bf16"), (100_000, 0, "f32")):
        idx = np.sort(rng.permutation(n)[:k]).astype(np.int32)
        val = wl.small_case("normal", max(k, 1), seed=k + 1, dtype=dtype)[:k]
        for off in (0, 1, 3):
            got = H.gpu_decompress(idx, val, n, off, sorted_call=True)
            assert np.array_equal(H.bits(got), H.bits(orc.decompress(idx, val, n))), (n, k, dtype, off)
    # clustered indices: all entries fall into one span, most spans have none
    n, k = 3_000_000, 20_000
    idx = (np.arange(k) + 1_234_567).astype(np.int32)
    val = wl.small_case("normal", k, seed=2)
    assert np.array_equal(H.bits(H.gpu_decompress(idx, val, n, 0, True)), H.bits(orc.decompress(idx, val, n)))
    # a caller that breaks the ascending-order promise gets a memory-safe call: every element written is
    # either zero or the value that belongs there (the harness checks the guard elements around the buffer)
    shuffled = rng.permutation(idx).astype(np.int32)
    got = H.gpu_decompress(shuffled, val, n, 0, True)
    full = orc.decompress(shuffled, val, n)
    assert np.all((H.bits(got) == 0) | (H.bits(got) == H.bits(full)))


def test_runs_are_bit_identical():
    import gpu_harness as H

    x = wl.small_case("few_levels", 1_000_003, seed=3)
    a = H.gpu_compress(x, 123_456)
    for _ in range(3):
        b = H.gpu_compress(x, 123_456)
        assert np.array_equal(a[0], b[0]) and np.array_equal(H.bits(a[1]), H.bits(b[1]))
        assert np.float32(a[2]).view(np.uint32) == np.float32(b[2]).view(np.uint32)


def test_segmented_mixed_lengths():
    import gpu_harness as H

    lens = [70_001, 0, 5, 8192, 1, 250_000, 16_384, 33]
    kinds = ["normal", "normal", "few_levels", "sparse", "normal", "few_levels", "all_equal", "nonfinite"]
    xs = [wl.small_case(kd, n, seed=40 + i) for i, (kd, n) in enumerate(zip(kinds, lens))]
    ks = [700, 0, 5, 100, 0, 40_000, 16_384, 11]
    gi, gv, off, ge = H.gpu_compress_segmented(xs, ks)
    ri, rv, roff, re = orc.compress_segmented(xs, ks)
    assert np.array_equal(off, roff) and np.array_equal(gi, ri) and np.array_equal(H.bits(gv), H.bits(rv))
    for s in range(len(xs)):
        assert H.same_err(ge[s], re[s], ERR_RTOL), (s, ge[s], re[s])
    check_segmented_decompress(gi, gv, off, lens)


def check_segmented_decompress(gi, gv, off, lens):
    import gpu_harness as H

    ys = H.gpu_decompress_segmented(gi, gv, off, lens)
    for s, n in enumerate(lens):
        ref = orc.decompress(gi[off[s]:off[s + 1]], gv[off[s]:off[s + 1]], n)
        assert np.array_equal(H.bits(ys[s]), H.bits(ref)), ("segmented decompress, tensor", s, n)


def test_segmented_more_segments_than_one_launch_holds():
    import gpu_harness as H

    rng = np.random.Generator(np.random.PCG64(17))
    lens = rng.integers(1, 30_000, size=70).tolist()
    for dtype in ("bf16", "f16"):
        xs = [wl.small_case("normal", n, seed=500 + i, dtype=dtype) for i, n in enumerate(lens)]
        ks = [max(1, n // 13) for n in lens]
        gi, gv, off, ge = H.gpu_compress_segmented(xs, ks)
        ri, rv, roff, re = orc.compress_segmented(xs, ks)
        assert np.array_equal(gi, ri) and np.array_equal(H.bits(gv), H.bits(rv))
        assert all(H.same_err(ge[s], re[s], ERR_RTOL) for s in range(len(xs)))
        check_segmented_decompress(gi, gv, off, lens)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_decompress_accumulate(dtype):
    import torch

    import gpu_harness as H
    from paper_2410_12707_amd import binding as B

    rng = np.random.Generator(np.random.PCG64(71))
    for n, k, kind in ((1, 1, "normal"), (70_001, 700, "normal"), (1_000_003, 1_000_003, "normal"),
                       (300_000, 40_000, "few_levels"), (50_000, 5_000, "nonfinite")):
        y = wl.small_case(kind, n, seed=72 + n, dtype=dtype)
        val = wl.small_case(kind, k, seed=73 + n, dtype=dtype)
        idx = rng.permutation(n)[:k].astype(np.int32)
        ref = orc.decompress_accumulate(idx, val, y)
        dy, dv = H.to_device(y, 1), H.to_device(val)
        B.adatopk_decompress_accumulate(torch.from_numpy(idx).cuda(), dv, k, dy)
        torch.cuda.synchronize()
        got = H.to_host(dy)
        if dtype == "f32":
            nan = np.isnan(ref)
            gnan = np.isnan(got)
        else:  # 16-bit: exponent all ones and a non-zero fraction
            frac = np.uint16(0x007F if dtype == "bf16" else 0x03FF)
            expo = np.uint16(0x7F80 if dtype == "bf16" else 0x7C00)
            nan = ((H.bits(ref) & expo) == expo) & ((H.bits(ref) & frac) != 0)
            gnan = ((H.bits(got) & expo) == expo) & ((H.bits(got) & frac) != 0)
        assert np.array_equal(nan, gnan), (dtype, n, k, kind)  # a NaN sum may carry any payload
        assert np.array_equal(H.bits(got)[~nan], H.bits(ref)[~nan]), (dtype, n, k, kind)
    # out-of-range indices are skipped, k = 0 is a no-op
    y = wl.small_case("normal", 1000, seed=1, dtype=dtype)
    dy = H.to_device(y)
    bad = np.array([-1, 1000, 5, 2_000_000_000], dtype=np.int32)
    val = wl.small_case("normal", 4, seed=2, dtype=dtype)
    B.adatopk_decompress_accumulate(torch.from_numpy(bad).cuda(), H.to_device(val), 4, dy)
    B.adatopk_decompress_accumulate(torch.from_numpy(bad).cuda(), H.to_device(val), 0, dy)
    torch.cuda.synchronize()
    assert np.array_equal(H.bits(H.to_host(dy)), H.bits(orc.decompress_accumulate(bad[2:3], val[2:3], y)))


def test_two_incoming_gradients_sum_like_the_oracle():
    # a node with two users (backward pass): compress each incoming gradient, accumulate both
    import torch

    import gpu_harness as H
    from paper_2410_12707_amd import binding as B

    n, k = 2_000_003, 20_000
    gs = [wl.small_case("normal", n, seed=80 + i) for i in range(2)]
    acc_ref = np.zeros(n, dtype=np.float32)
    acc = torch.zeros(n, dtype=torch.float32, device="cuda")
    ws = B.new_workspace(n, 1, torch.float32)
    for g in gs:
        ri, rv, _ = orc.compress(g, k)
        acc_ref = orc.decompress_accumulate(ri, rv, acc_ref)
        idx = torch.empty(k, dtype=torch.int32, device="cuda")
        val = torch.empty(k, dtype=torch.float32, device="cuda")
        B.adatopk_compress(H.to_device(g), k, idx, val, None, ws)
        B.adatopk_decompress_accumulate(idx, val, k, acc)
    torch.cuda.synchronize()
    assert np.array_equal(H.bits(H.to_host(acc)), H.bits(acc_ref))


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("limit", [8192, 65_536])
def test_many_small_tensors_in_one_call(dtype, limit):
    # the launch-bound regime: hundreds of small messages in one call.  With every tensor within
    # 8192 elements the one-launch path takes them (more than one of its launches holds); with
    # larger ones in the mix the four-kernel path batches them, several launches as well
    import gpu_harness as H

    rng = np.random.Generator(np.random.PCG64(23))
    lens = [1, 63, 64, 65, 511, 512, 513, 1023, 1024, 1025, 4095, 4096, 4097, 8191, 8192, 0]
    if limit > 8192:
        lens += [8193, 16384, 32768, 65535, 65536]
    lens += rng.integers(1, limit + 1, size=300 - len(lens)).tolist()
    kinds = ["normal", "few_levels", "sparse", "all_equal", "nonfinite", "random_bits", "signed_zero_mix"]
    xs = [wl.small_case(kinds[i % len(kinds)], n, seed=900 + i, dtype=dtype) for i, n in enumerate(lens)]
    ks = [int(rng.integers(0, n + 1)) if i % 3 else max(0, n // 100) for i, n in enumerate(lens)]
    gi, gv, off, ge = H.gpu_compress_segmented(xs, ks)
    ri, rv, roff, re = orc.compress_segmented(xs, ks)
    assert np.array_equal(off, roff) and np.array_equal(gi, ri) and np.array_equal(H.bits(gv), H.bits(rv))
    for s in range(len(xs)):
        assert H.same_err(ge[s], re[s], ERR_RTOL), (s, lens[s], ks[s], ge[s], re[s])
    check_segmented_decompress(gi, gv, off, lens)


def test_small_tensor_limit_and_one_past_it():
    for n in (8192, 8193):  # the last size of the one-launch path and the first of the four-kernel path
        for kind in ("few_levels", "normal"):
            x = wl.small_case(kind, n, seed=n)
            for k in (1, n // 7, n - 1, n):
                check_one(x, k, label="%s n=%d k=%d" % (kind, n, k))


def test_randomized_shapes_and_keep_counts():
    # 160 seeded draws of (dtype, value structure, n, k): n log-uniform from 1 to 400 000, so both compress
    # paths, one to several chunks and list blocks, k anywhere from 0 to n
    rng = np.random.Generator(np.random.PCG64(2410_12707))
    kinds = ["normal", "few_levels", "sparse", "all_equal", "random_bits", "signed_zero_mix", "nonfinite", "ascending"]
    for case in range(160):
        dtype = ["f32", "bf16", "f16"][case % 3]
        kind = kinds[int(rng.integers(0, len(kinds)))]
        n = int(np.exp(rng.uniform(0.0, np.log(400_000.0))))
        k = int(rng.integers(0, n + 1)) if case % 2 else int(n * np.exp(rng.uniform(np.log(1e-3), 0.0)))
        x = wl.small_case(kind, n, seed=5000 + case, dtype=dtype)
        check_one(x, k, label="case %d: %s %s n=%d k=%d" % (case, kind, dtype, n, k))


@pytest.mark.parametrize("n", [5000, 300_000])
def test_error_norm_is_optional(n):
    # err_norm_out = NULL: same indices and values, on the one-launch path (n <= 8192) and the four-kernel path,
    # single and segmented
    import gpu_harness as H

    x = wl.small_case("normal", n, seed=n)
    k = n // 20
    ri, rv, _ = orc.compress(x, k)
    gi, gv, ge = H.gpu_compress(x, k, want_err=False)
    assert ge is None and np.array_equal(gi, ri) and np.array_equal(H.bits(gv), H.bits(rv))
    xs = [x, wl.small_case("few_levels", n // 2, seed=n + 1)]
    ks = [k, n // 8]
    si, sv, off, se = H.gpu_compress_segmented(xs, ks, want_err=False)
    qi, qv, qoff, _ = orc.compress_segmented(xs, ks)
    assert se is None and np.array_equal(si, qi) and np.array_equal(H.bits(sv), H.bits(qv))


def _sampled_elements(n, esize):
    """Element indices that the speculative scan may look at before it reads the tensor: runs of 1 KB,
    evenly spaced with a small run-dependent shift, for each of its sample sizes (mirrors the kernel's
    sampling on purpose: the test below plants values exactly there)."""
    dwords = n * esize // 4
    nruns = dwords // 256
    idx = []
    for nbatch in ((1, 2, 4) if esize == 4 else (1, 2)):
        runs = nbatch * 4 * 8
        shift = runs.bit_length() - 1
        for r in range(runs):
            run = ((r * (nruns - 32)) >> shift) + (r * 37) % 32
            first = run * 1024 // esize
            idx.append(np.arange(first, first + 1024 // esize))
    return np.unique(np.concatenate(idx))


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("scale", [64.0, 1.0 / 64.0])
def test_speculation_misled_by_its_sample_falls_back_to_the_exact_select(dtype, scale):
    # The one-read path brackets the k-th key from a sample and must never be trusted: here the sampled
    # places hold values 64 times larger (the bracket lands far above the k-th key: too few candidates) or
    # 64 times smaller (far below: the k-th key falls into the window's open-ended last bin) than the rest
    # of the tensor.  The exact passes behind the speculative scan have to notice and redo the selection.
    import torch

    import gpu_harness as H
    from paper_2410_12707_amd import binding as B

    n, k = 4_200_003, 42_000
    esize = 4 if dtype == "f32" else 2
    x = wl.small_case("normal", n, seed=321, dtype="f32")
    at = _sampled_elements(n, esize)
    x[at] *= np.float32(scale)
    if dtype == "bf16":
        x = wl.f32_to_bf16_bits(x)
    elif dtype == "f16":
        x = x.astype(np.float16)
    # (a 16-bit window spans 2047 patterns, 16 binades of bf16 but two of fp16, upwards of its lowest key:
    # a bracket that is 64 times too low still contains the k-th key in bf16, at the price of candidate
    # lists that overflow)
    misled = 1 if (dtype == "bf16" and scale < 1.0) else 0
    for data, expect_held in ((x, misled), (wl.small_case("normal", n, seed=321, dtype=dtype), 1)):
        d = H.to_device(data)
        idx = torch.full((k,), -7, dtype=torch.int32, device="cuda")
        val = torch.zeros(k, dtype=d.dtype, device="cuda")
        err = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
        ws = B.new_workspace(n, 1, d.dtype)
        B.adatopk_compress(d, k, idx, val, err, ws)
        torch.cuda.synchronize()
        # the tensor's state record opens the workspace; its seventh word says whether the speculation held
        held = int(ws[:64].view(torch.int32)[6].item())
        assert held == expect_held, (dtype, scale, held)
        ri, rv, re = orc.compress(data, k)
        assert np.array_equal(H.to_host(idx), ri) and np.array_equal(H.bits(H.to_host(val)), H.bits(rv))
        assert H.same_err(H.to_host(err)[0], re, ERR_RTOL)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_midsize_tensors_value_structures_and_boundaries(dtype):
    # between the one-launch path for small tensors and the sizes at which a sample of the tensor is taken
    # first (2^20 elements): the exact two-pass select with tens to hundreds of chunks, around powers of two,
    # with value structures whose candidate lists overflow (constant, few levels), keep counts of 0 and 1
    for n, k in ((65_535, 600), (65_536, 655), (65_537, 1), (300_000, 6144), (300_000, 6145), (1_048_575, 6000),
                 (1_048_576, 6000), (1_048_577, 6000), (524_288, 0), (200_001, 2000)):
        for kind in ("normal", "few_levels", "all_equal", "sparse", "descending", "nonfinite"):
            check_one(wl.small_case(kind, n, seed=n % 1000 + k, dtype=dtype), k, label="%s %s n=%d k=%d" % (kind, dtype, n, k))


def test_midsize_tensors_in_one_segmented_call():
    import gpu_harness as H

    lens = [70_000, 0, 8192, 150_001, 65_536, 9_000, 400_000, 1, 262_144]
    kinds = ["normal", "normal", "few_levels", "sparse", "normal", "all_equal", "normal", "normal", "descending"]
    xs = [wl.small_case(kd, n, seed=60 + i) for i, (kd, n) in enumerate(zip(kinds, lens))]
    ks = [700, 0, 8192, 1500, 650, 90, 4000, 1, 0]
    gi, gv, off, ge = H.gpu_compress_segmented(xs, ks)
    ri, rv, roff, re = orc.compress_segmented(xs, ks)
    assert np.array_equal(off, roff) and np.array_equal(gi, ri) and np.array_equal(H.bits(gv), H.bits(rv))
    for s in range(len(xs)):
        assert H.same_err(ge[s], re[s], ERR_RTOL), (s, ge[s], re[s])
    check_segmented_decompress(gi, gv, off, lens)
