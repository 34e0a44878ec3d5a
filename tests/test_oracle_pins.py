"""Pins of the CPU oracle against things other than itself (CPU only).

The paper prints no worked numeric example of the Top-K step (its illustration is a
figure), so the selection is pinned by the definition in Sec. 5.1 (the k entries of
largest absolute value are sent as (index, value) pairs, the rest decompress to 0):
brute force, exhaustive subsets, invariants, library special cases and closed forms.
The error norm is pinned by an fp64 identity and by the Gaussian closed form; the ratio
rule by Eq. "adacompress" (Sec. 5.2) worked by hand, and by the wire-size arithmetic the
paper prints (tests/golden/).
"""
import itertools
import json
import math
import os

import numpy as np
import pytest

from oracle import adatopk_oracle as orc
from paper_2410_12707_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers
def magnitudes(x):
    """|x| as float64 for finite inputs (fp32 or fp16 array, or uint16 bf16 bit patterns)."""
    if x.dtype == np.uint16:
        x = wl.bf16_bits_to_f32(x)
    return np.abs(x.astype(np.float64))


def brute_force_topk(mag, k):
    """k rounds of: scan for the largest magnitude, first occurrence wins, remove it."""
    mag = list(mag)
    taken = []
    alive = [True] * len(mag)
    for _ in range(k):
        best = -1
        for i, m in enumerate(mag):
            if alive[i] and (best < 0 or m > mag[best]):
                best = i
        alive[best] = False
        taken.append(best)
    return sorted(taken)


def bits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a.view(np.uint16)


KINDS = ["normal", "few_levels", "all_equal", "sparse", "signed_zero_mix", "descending", "ascending"]


# ----------------------------------------------------------------------- brute force
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("kind", KINDS)
def test_selection_matches_repeated_argmax(kind, dtype):
    for n in (1, 2, 7, 64, 193):
        x = wl.small_case(kind, n, seed=100 + n, dtype=dtype)
        mag = magnitudes(x)
        for k in sorted({0, 1, n // 3, n - 1, n} - {-1}):
            if k < 0:
                continue
            idx, val, _ = orc.compress(x, k)
            assert idx.tolist() == brute_force_topk(mag, k), (kind, dtype, n, k)
            assert np.array_equal(bits(val), bits(x)[idx])


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_selection_is_optimal_and_lexicographically_first_over_all_subsets(dtype):
    # For n <= 10 enumerate every k-subset: the chosen one must have the largest multiset
    # of magnitudes (compared as sorted-descending tuples) and, among those, the smallest
    # sorted index tuple.
    for seed, kind in enumerate(["few_levels", "normal", "sparse", "few_levels"]):
        n = 7 + seed
        x = wl.small_case(kind, n, seed=900 + seed, dtype=dtype)
        mag = magnitudes(x)
        for k in range(0, n + 1):
            best = None
            for sub in itertools.combinations(range(n), k):
                score = (tuple(sorted((mag[i] for i in sub), reverse=True)), tuple(-i for i in sub))
                if best is None or score > best[0]:
                    best = (score, sub)
            idx, _, _ = orc.compress(x, k)
            assert tuple(idx.tolist()) == best[1], (kind, n, k)


def test_hypothesis_small_arrays_against_brute_force():
    # hypothesis searches small arrays (drawn from a small value set, so ties are the rule) for a case
    # where the oracle departs from the repeated arg-max; derandomised, so every run tries the same cases
    from hypothesis import given, settings
    from hypothesis import strategies as st

    levels = [0.0, -0.0, 0.5, -0.5, 1.0, -1.0, 1.5, 2.0, -2.0, 1e-40, float("inf"), -float("inf")]

    @settings(max_examples=300, deadline=None, derandomize=True)
    @given(st.lists(st.sampled_from(levels), min_size=1, max_size=24), st.data())
    def run(values, data):
        x = np.array(values, dtype=np.float32)
        k = data.draw(st.integers(min_value=0, max_value=x.size))
        idx, val, _ = orc.compress(x, k)
        key = (x.view(np.uint32) & np.uint32(0x7FFFFFFF)).astype(np.int64)  # orders Inf and denormals too
        assert idx.tolist() == brute_force_topk(key, k)
        assert np.array_equal(val.view(np.uint32), x.view(np.uint32)[idx])
        y = orc.decompress(idx, val, x.size)
        keep = np.zeros(x.size, dtype=bool)
        keep[idx] = True
        assert np.array_equal(y.view(np.uint32), np.where(keep, x.view(np.uint32), 0))

    run()


# ------------------------------------------------------------------------- invariants
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("kind", ["normal", "few_levels", "sparse", "nonfinite", "random_bits"])
def test_selection_invariants(kind, dtype):
    n = 50_021
    x = wl.small_case(kind, n, seed=7, dtype=dtype)
    sign_clear = np.uint32(0x7FFFFFFF) if dtype == "f32" else np.uint16(0x7FFF)
    key = bits(x) & sign_clear
    for k in (1, 500, n // 2, n - 1):
        idx, val, _ = orc.compress(x, k)
        assert idx.dtype == np.int32 and idx.size == k
        assert np.all(np.diff(idx.astype(np.int64)) > 0) and idx[0] >= 0 and idx[-1] < n
        assert np.array_equal(bits(val), bits(x)[idx])
        mask = np.zeros(n, dtype=bool)
        mask[idx] = True
        kmin = key[mask].min()
        assert kmin >= key[~mask].max()
        # lowest index wins among elements that tie with the smallest kept key
        tied_dropped = np.nonzero(~mask & (key == kmin))[0]
        tied_kept = np.nonzero(mask & (key == kmin))[0]
        if tied_dropped.size:
            assert tied_kept.max() < tied_dropped.min()


# ---------------------------------------------------------- library special cases
def test_distinct_magnitudes_agree_with_numpy_and_torch():
    import torch

    rng = np.random.Generator(np.random.PCG64(5))
    n = 20_000
    # distinct magnitudes by construction: a permutation of 1..n scaled, random signs
    x = (rng.permutation(n).astype(np.float32) + 1.0) * np.float32(0.125)
    x *= rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=n)
    for k in (1, 17, 2_000, n - 1, n):
        idx, _, _ = orc.compress(x, k)
        ref_np = np.sort(np.argsort(-np.abs(x), kind="stable")[:k])
        ref_t = torch.topk(torch.from_numpy(x).abs(), k).indices.sort().values.numpy()
        assert np.array_equal(idx, ref_np)
        assert np.array_equal(idx, ref_t)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_lexsort_statement_of_the_definition(dtype):
    # Same definition through numpy's lexsort (key descending, index ascending), with ties.
    for kind in ("few_levels", "normal", "sparse"):
        n = 30_011
        x = wl.small_case(kind, n, seed=11, dtype=dtype)
        mag = magnitudes(x)
        order = np.lexsort((np.arange(n), -mag))
        for k in (3, 999, n // 2):
            idx, _, _ = orc.compress(x, k)
            assert np.array_equal(idx, np.sort(order[:k]))


# ---------------------------------------------------------------------- closed forms
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_closed_forms(dtype):
    n = 1000
    eq = wl.small_case("all_equal", n, 0, dtype)
    for k in (1, 10, n):
        idx, val, err = orc.compress(eq, k)
        assert np.array_equal(idx, np.arange(k))
        assert math.isclose(float(err), 1.5 * math.sqrt(n - k), rel_tol=1e-6)
    x = wl.small_case("normal", n, 3, dtype)
    idx, val, err = orc.compress(x, n)  # k = n is the identity
    assert np.array_equal(idx, np.arange(n)) and np.array_equal(bits(val), bits(x)) and float(err) == 0.0
    idx, val, _ = orc.compress(x, 1)  # k = 1: first occurrence of the largest magnitude
    assert idx[0] == int(np.argmax(magnitudes(x)))
    idx, val, err = orc.compress(x, 0)  # k = 0: nothing kept, everything is error
    assert idx.size == 0 and math.isclose(float(err), math.sqrt(float(np.sum(magnitudes(x) ** 2))), rel_tol=1e-6)
    d = wl.small_case("descending", 200, 0, dtype)  # distinct and exactly representable in bf16 up to 256
    assert np.array_equal(orc.compress(d, 20)[0], np.arange(20))
    a = wl.small_case("ascending", 200, 0, dtype)
    assert np.array_equal(orc.compress(a, 20)[0], np.arange(180, 200))


def test_negative_values_rank_by_magnitude_and_keep_their_sign():
    x = np.array([0.5, -3.0, 2.0, -0.25, 3.0, -2.5], dtype=np.float32)
    idx, val, err = orc.compress(x, 3)
    assert idx.tolist() == [1, 4, 5]
    assert val.tolist() == [-3.0, 3.0, -2.5]
    assert math.isclose(float(err), math.sqrt(0.25 + 4.0 + 0.0625), rel_tol=1e-7)
    idx, _, _ = orc.compress(x, 1)  # |-3| ties with |3|: lowest index
    assert idx.tolist() == [1]


def test_nonfinite_ordering_and_bit_exact_values():
    u = np.array([0x3F800000, 0x7F800000, 0xFFC01234, 0x00000001, 0x80000000, 0x7FC00000, 0xFF800000], dtype=np.uint32)
    x = u.view(np.float32)
    # keys: NaN payload 0x7FC01234 > NaN 0x7FC00000 > Inf (two of them, index order) > 1.0 > denormal > -0
    idx, val, _ = orc.compress(x, 4)
    assert idx.tolist() == [1, 2, 5, 6]
    assert np.array_equal(val.view(np.uint32), u[[1, 2, 5, 6]])
    idx, val, _ = orc.compress(x, 6)
    assert idx.tolist() == [0, 1, 2, 3, 5, 6]
    assert val.view(np.uint32)[3] == 1  # denormal kept bit-exact (no flush to zero)


def test_fp16_widening_matches_numpy_for_every_pattern():
    # The oracle widens binary16 by the format's definition; numpy's float16 is the independent reading.
    pats = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    ref = pats.view(np.float16).astype(np.float32)
    got = np.array([orc.f16_to_f32(int(p)) for p in pats], dtype=np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def test_fp16_denormals_extremes_and_hand_error():
    # 2^-24 (smallest denormal), 2^-14 (smallest normal), 65504 (largest finite), -Inf, -2^-24
    u = np.array([0x0001, 0x0400, 0x7BFF, 0xFC00, 0x8001], dtype=np.uint16)
    x = u.view(np.float16)
    idx, val, err = orc.compress(x, 2)
    assert idx.tolist() == [2, 3] and val.view(np.uint16).tolist() == [0x7BFF, 0xFC00]
    assert math.isclose(float(err), math.sqrt(2.0 ** -48 + 2.0 ** -28 + 2.0 ** -48), rel_tol=1e-7)
    idx, _, err = orc.compress(x, 4)  # the two denormals tie: lowest index
    assert idx.tolist() == [0, 1, 2, 3] and math.isclose(float(err), 2.0 ** -24, rel_tol=1e-7)


# -------------------------------------------------------------------- reconstruction
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("kind", ["normal", "few_levels", "nonfinite"])
def test_decompress_is_the_masked_input(kind, dtype):
    n = 10_007
    x = wl.small_case(kind, n, seed=21, dtype=dtype)
    for k in (0, 1, 100, n):
        idx, val, _ = orc.compress(x, k)
        y = orc.decompress(idx, val, n)
        mask = np.zeros(n, dtype=bool)
        mask[idx] = True
        expect = np.where(mask, bits(x), 0).astype(bits(x).dtype)  # +0.0 is the all-zero pattern
        assert np.array_equal(bits(y), expect)
        if k and kind != "nonfinite":
            idx2, val2, _ = orc.compress(y, k)  # idempotent while the smallest kept magnitude is non-zero
            if magnitudes(val).min() > 0:
                assert np.array_equal(idx2, idx) and np.array_equal(bits(val2), bits(val))


def test_decompress_accepts_any_order_and_rejects_out_of_range():
    idx = np.array([5, 0, 3], dtype=np.int32)
    val = np.array([1.0, -2.0, 3.0], dtype=np.float32)
    assert orc.decompress(idx, val, 6).tolist() == [-2.0, 0.0, 0.0, 3.0, 0.0, 1.0]
    with pytest.raises(ValueError):
        orc.decompress(np.array([6], dtype=np.int32), val[:1], 6)


# ---------------------------------------------------------------- accumulating decompress
def test_rounding_to_fp16_matches_numpy_on_ties_and_random_values():
    pats = np.arange(0x7C00, dtype=np.uint32).astype(np.uint16)  # every non-negative finite value, ascending
    v = pats.view(np.float16).astype(np.float64)
    mids = (v[:-1] + v[1:]) / 2  # exact in fp64: the ties between neighbours
    rng = np.random.Generator(np.random.PCG64(61))
    rnd = rng.standard_normal(20000) * np.exp(rng.uniform(-20, 12, 20000))
    probe = np.concatenate([v, mids, np.nextafter(mids, 0), np.nextafter(mids, np.inf), rnd, [65519.9, 65520.0, 1e9]])
    probe = np.concatenate([probe, -probe])
    with np.errstate(over="ignore"):
        ref = probe.astype(np.float16).view(np.uint16)
    got = np.array([orc.round_f16(float(t)) for t in probe], dtype=np.uint16)
    assert np.array_equal(got, ref)


def test_rounding_to_bf16_matches_torch_on_ties_and_random_values():
    import torch

    rng = np.random.Generator(np.random.PCG64(62))
    pats = rng.integers(0, 0x7F7F, size=4000, dtype=np.uint32).astype(np.uint16)  # finite bf16 values
    lo = wl.bf16_bits_to_f32(pats).astype(np.float64)
    hi = wl.bf16_bits_to_f32(pats + np.uint16(1)).astype(np.float64)
    mids = ((lo + hi) / 2).astype(np.float32)  # ties are fp32 values: one more bit than bf16
    rnd = (rng.standard_normal(20000) * np.exp(rng.uniform(-80, 80, 20000))).astype(np.float32)
    probe = np.concatenate([mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(np.inf)), rnd,
                            np.array([3.3895e38, 3.4e38, 1e-40, 4.6e-41, 0.0], dtype=np.float32)])
    probe = np.concatenate([probe, -probe])
    ref = torch.from_numpy(probe).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([orc.round_bf16(float(t)) for t in probe], dtype=np.uint16)
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_accumulate_matches_library_addition(dtype):
    import torch

    n, k = 20_011, 3_000
    rng = np.random.Generator(np.random.PCG64(63))
    y = wl.small_case("normal", n, seed=64, dtype=dtype)
    val = wl.small_case("normal", k, seed=65, dtype=dtype)
    idx = rng.permutation(n)[:k].astype(np.int32)
    got = orc.decompress_accumulate(idx, val, y)
    if dtype == "bf16":
        t = torch.from_numpy(y.view(np.int16).copy()).view(torch.bfloat16)
        t[torch.from_numpy(idx.astype(np.int64))] += torch.from_numpy(val.view(np.int16).copy()).view(torch.bfloat16)
        ref = t.view(torch.int16).numpy().view(np.uint16)
    else:
        ref = y.copy()
        ref[idx] += val  # numpy's own addition in the type
    assert np.array_equal(bits(got), bits(ref))
    untouched = np.ones(n, dtype=bool)
    untouched[idx] = False
    assert np.array_equal(bits(got)[untouched], bits(y)[untouched])


def test_accumulate_hand_examples_and_sum_of_two_messages():
    # bf16 has 8 significand bits: 1 + 2^-8 is a tie and goes to even (1.0); 1 + 2^-7 + 2^-8 goes up to 1 + 2^-6
    y = np.array([0x3F80, 0x3F81, 0x7F7F, 0x0001, 0x3F80], dtype=np.uint16)  # 1, 1+2^-7, max finite, min denormal, 1
    v = np.array([0x3B80, 0x3B80, 0x7F7F, 0x0001, 0xBF80], dtype=np.uint16)  # 2^-8, 2^-8, max finite, min denormal, -1
    out = orc.decompress_accumulate(np.arange(5, dtype=np.int32), v, y)
    assert out.tolist() == [0x3F80, 0x3F82, 0x7F80, 0x0002, 0x0000]
    # fp16: 2048 + 1 is a tie (spacing 2 there) and goes to even 2048; 2050 + 1 goes up to 2052; 65504 + 32 overflows
    yh = np.array([2048.0, 2050.0, 65504.0, 6e-8], dtype=np.float16)
    vh = np.array([1.0, 1.0, 32.0, 6e-8], dtype=np.float16)
    outh = orc.decompress_accumulate(np.arange(4, dtype=np.int32), vh, yh)
    assert outh[:2].tolist() == [2048.0, 2052.0] and np.isinf(outh[2]) and outh.view(np.uint16)[3] == 2
    # a node with two users: the two compressed gradients add up where both kept an entry
    n = 1000
    g1 = np.zeros(n, dtype=np.float32)
    g2 = np.zeros(n, dtype=np.float32)
    g1[[3, 500, 999]] = [4.0, -2.0, 8.0]
    g2[[3, 7, 999]] = [0.5, 16.0, -8.0]
    acc = np.zeros(n, dtype=np.float32)
    for g in (g1, g2):
        idx, val, _ = orc.compress(g, 3)
        acc = orc.decompress_accumulate(idx, val, acc)
    assert np.array_equal(acc, g1 + g2)
    with pytest.raises(ValueError):
        orc.decompress_accumulate(np.array([n], dtype=np.int32), np.ones(1, np.float32), acc)


# ------------------------------------------------------------------------ error norm
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_error_norm_identity_in_fp64(dtype):
    n = 200_003
    x = wl.small_case("normal", n, seed=33, dtype=dtype)
    tot = float(np.sum(magnitudes(x) ** 2))
    for k in (1, n // 100, n // 3):
        idx, val, err = orc.compress(x, k)
        kept = float(np.sum(magnitudes(val) ** 2))
        assert err.dtype == np.float32
        assert math.isclose(float(err), math.sqrt(tot - kept), rel_tol=2e-7)


def test_error_norm_gaussian_closed_form():
    # For i.i.d. N(0,1) and keep fraction rho, the dropped energy fraction tends to
    # 1 - 2 [ t phi(t) + 1 - Phi(t) ] with t = Phi^{-1}(1 - rho/2).
    from scipy.stats import norm

    n = 4_000_000
    x = wl.normal_f32(n, seed=44)
    rho = 0.01
    t = norm.ppf(1 - rho / 2)
    expect = math.sqrt(1 - 2 * (t * norm.pdf(t) + 1 - norm.cdf(t)))
    idx, val, err = orc.compress(x, int(n * rho))
    rel = float(err) / math.sqrt(float(np.sum(x.astype(np.float64) ** 2)))
    assert abs(rel - expect) < 2e-3
    assert abs(float(np.min(np.abs(val))) - t) < 2e-2  # the threshold is the (1 - rho/2) quantile


# --------------------------------------------------------------------------- segmented
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_segmented_is_per_tensor(dtype):
    # Unequal lengths, an empty tensor in the middle and at the end, lengths 1 and 2, k = 0 and k = n.
    # Every tensor's part of the output is checked against the repeated arg-max on that tensor alone
    # (so a wrong input or output offset, or a k taken from the neighbour, shows) and against the
    # single-tensor routine, error norm included.
    kinds = ["normal", "few_levels", "sparse", "normal", "all_equal", "normal", "few_levels", "normal"]
    ns = [500, 129, 1, 0, 2, 193, 64, 0]
    ks = [50, 129, 0, 0, 1, 7, 0, 0]
    xs = [wl.small_case(kind, n, 300 + s, dtype=dtype) if n else wl.small_case("normal", 1, 1, dtype=dtype)[:0]
          for s, (kind, n) in enumerate(zip(kinds, ns))]
    idx, val, off, err = orc.compress_segmented(xs, ks)
    assert off.tolist() == [0, 50, 179, 179, 179, 180, 187, 187, 187]
    assert idx.size == 187 and val.size == 187 and err.size == len(xs) and val.dtype == xs[0].dtype
    for s, (x, k) in enumerate(zip(xs, ks)):
        part_i, part_v = idx[off[s]:off[s + 1]], val[off[s]:off[s + 1]]
        assert part_i.tolist() == brute_force_topk(magnitudes(x), k), (dtype, s)
        assert np.array_equal(bits(part_v), bits(x)[part_i])
        keep = np.zeros(x.size, dtype=bool)
        keep[part_i] = True
        dropped = float(np.sum(magnitudes(x)[~keep] ** 2))
        assert math.isclose(float(err[s]), math.sqrt(dropped), rel_tol=2e-7, abs_tol=0.0)
        i1, v1, e1 = orc.compress(x, k)
        assert np.array_equal(part_i, i1) and np.array_equal(bits(part_v), bits(v1)) and err[s] == e1


# ------------------------------------------------------------- ratio rule and wire size
def test_adaptive_ratio_rule_hand_example():
    with open(os.path.join(GOLDEN, "adacompress_hand_example.json")) as f:
        g = json.load(f)
    for case in g["cases"]:
        out = orc.adaptive_ratios(case["R"], case["r"], case["coeff"])
        assert np.allclose(out, case["r_i"], rtol=1e-12, atol=0)


def test_wire_size_arithmetic_printed_in_the_paper():
    with open(os.path.join(GOLDEN, "wire_size.json")) as f:
        g = json.load(f)
    # Top-K figure caption: a d-vector of 32-bit values (32 d bits) becomes k values plus k
    # 32-bit indices (64 k bits).
    d, k = 1_000_000, orc.k_for_ratio(1_000_000, g["ratio"])
    assert k == d // g["ratio"]
    # the oracle's message of k pairs (fp32 values, int32 indices) carries exactly the caption's 64 bits
    # per kept element behind its fixed header, against the caption's 32 bits per element of the dense vector
    from oracle import wire_format as wf

    payload_bits = 8 * (wf.message_bytes(k, np.float32, 4) - wf.message_bytes(0, np.float32, 4))
    assert payload_bits == g["fig_topk_wire_bits_per_kept"] * k
    assert 8 * np.dtype(np.float32).itemsize == g["fig_topk_dense_bits_per_element"]
    # Latency figure caption: at ratio 100 with fp32 values and int64 indices the data sent
    # is 33.3x smaller; the same accounting gives the coefficient 3 of Eq. "adacompress".
    shrink = (4 * d) / ((4 + 8) * k)
    assert abs(shrink - g["latency_fig_shrink_at_ratio_100"]) < 0.05
    assert (4 + 8) / 4 == g["adacompress_coefficient"]


def test_k_for_ratio_rounding():
    assert orc.k_for_ratio(393_216, 100.0) == 3_932  # 1 % of the GPT-2-small tensor, floor
    assert orc.k_for_ratio(1000, 1.0) == 1000  # ratio 1: no compression
    assert orc.k_for_ratio(1000, 3000.0) == 1  # never fewer than one element
    assert orc.k_for_ratio(0, 10.0) == 0
    assert orc.k_for_ratio(10, 0.5) == -1  # a ratio below 1 is not a compression ratio


# ------------------------------------------- link model and pipeline-time estimates (Sec. 3.5, 3.6, 5.2)
def test_link_and_pipeline_estimates_hand_example():
    with open(os.path.join(GOLDEN, "pipeline_hand_example.json")) as f:
        g = json.load(f)
    ln, pp = g["link"], g["pipeline"]
    assert math.isclose(orc.link_time(ln["alpha"], ln["beta"], ln["bytes"]), ln["T"], rel_tol=1e-12)
    assert math.isclose(orc.pipeline_time(pp["C"], pp["R"], pp["n_b"]), pp["time_pipe"], rel_tol=1e-12)
    assert np.allclose(orc.adaptive_ratios(pp["R"], pp["r"], pp["coeff"]), pp["r_i"], rtol=1e-12)
    assert math.isclose(orc.pipeline_time_compressed(pp["C"], pp["R"], pp["n_b"], pp["r"], pp["coeff"], 0),
                        pp["time_pipe_compress_printed"], rel_tol=1e-12)
    assert math.isclose(orc.pipeline_time_compressed(pp["C"], pp["R"], pp["n_b"], pp["r"], pp["coeff"], 1),
                        pp["time_pipe_compress_own_ratio"], rel_tol=1e-12)
    # special cases that follow from the equations: one micro-batch has no bottleneck term; ratio 1/coeff
    # on equal links sends exactly the uncompressed volume
    C, R = [0.3, 0.7], [2.0, 2.0]
    assert math.isclose(orc.pipeline_time(C, R, 1), 5.0, rel_tol=1e-12)
    assert math.isclose(orc.pipeline_time_compressed(C, R, 1, 1.0 / 3.0 * 3.0, 3.0, 1),
                        orc.pipeline_time(C, [r_ * 3.0 / 3.0 for r_ in R], 1), rel_tol=1e-12)
    pl = g["plan"]
    Rs = [orc.link_time(a, b, 4.0 * n) for a, b, n in zip(pl["alpha"], pl["beta"], pl["n"])]
    assert np.allclose(Rs, pl["R"], rtol=1e-12)
    ri = orc.adaptive_ratios(Rs, pl["r"], pl["coeff"])
    assert np.allclose(ri, pl["r_i"], rtol=1e-12)
    assert [orc.k_for_ratio(n, r) for n, r in zip(pl["n"], ri)] == pl["k"]
