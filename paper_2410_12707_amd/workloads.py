"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws numbers: it holds none of the compressor's arithmetic and is the
one module that both the CPU oracle's tests and the HIP path's tests / benchmark import.
The tensors stand in for the ResNet-101 and GPT-2 activations and activation gradients
that cross pipeline cuts in the paper's experiments (Sec. 7, model settings table);
the datasets and trained weights themselves are not used.

Every generator returns host numpy arrays: float32, uint16 holding bf16 bit
patterns, or float16.  Seeds are ``12707 + config number`` (config 4 adds ``100 * segment``).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

BASE_SEED = 12707


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def normal_f32(n: int, seed: int) -> np.ndarray:
    return _rng(seed).standard_normal(n, dtype=np.float32)


def gelu_of_normal_f32(n: int, seed: int) -> np.ndarray:
    """GELU(z), z ~ N(0,1), erf form, evaluated in fp32 (post-activation GPT-2 tensor)."""
    from scipy.special import erf

    z = normal_f32(n, seed)
    out = np.empty_like(z)
    step = 1 << 22
    inv_sqrt2 = np.float32(0.7071067811865476)
    for a in range(0, n, step):
        zz = z[a:a + step]
        out[a:a + step] = np.float32(0.5) * zz * (np.float32(1.0) + erf(zz * inv_sqrt2).astype(np.float32))
    return out


def student_t_f32(n: int, seed: int, dof: float = 3.0, scale: float = 1e-3) -> np.ndarray:
    """Heavy-tailed activation gradient: scale * Student-t(dof)."""
    rng = _rng(seed)
    out = np.empty(n, dtype=np.float32)
    step = 1 << 22
    for a in range(0, n, step):
        m = min(step, n - a)
        out[a:a + m] = (rng.standard_t(dof, size=m) * scale).astype(np.float32)
    return out


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(n: int, seed: int) -> np.ndarray:
    return f32_to_bf16_bits(normal_f32(n, seed))


def normal_f16(n: int, seed: int) -> np.ndarray:
    return normal_f32(n, seed).astype(np.float16)


@dataclass
class Workload:
    """One benchmark configuration: a list of tensors with one k each."""

    name: str
    dtype: str  # "f32" | "bf16" | "f16"
    shape: tuple
    tensors: List[np.ndarray] = field(default_factory=list)
    ks: List[int] = field(default_factory=list)
    note: str = ""
    # For workloads whose keep counts are to be PLANNED from link parameters (ks is then empty):
    # latency in seconds and inverse bandwidth in seconds per byte of the link each tensor crosses,
    # the user's ratio r and the coefficient of Eq. "adacompress".  Inputs only: the rule itself is
    # applied by whoever consumes the workload (the library on one side, the oracle on the other).
    alpha: List[float] = field(default_factory=list)
    beta: List[float] = field(default_factory=list)
    r_user: float = 0.0
    coeff: float = 0.0

    @property
    def n_total(self) -> int:
        return int(sum(t.size for t in self.tensors))


def keep_count(n: int, num: int, den: int) -> int:
    """k for a rational keep fraction num/den, in integer arithmetic (floor)."""
    return (n * num) // den


def config1() -> Workload:
    n = 4 * 128 * 768
    return Workload("cfg1_gpt2s_hidden_4x128x768_f32_k1pct", "f32", (4, 128, 768),
                    [normal_f32(n, BASE_SEED + 1)], [keep_count(n, 1, 100)],
                    "GPT-2-small hidden activation, N(0,1)")


def config2(keep=(1, 100)) -> Workload:
    n = 32 * 1024 * 768
    num, den = keep
    return Workload("cfg2_gpt2s_gelu_32x1024x768_f32_k%d_%d" % (num, den), "f32", (32, 1024, 768),
                    [gelu_of_normal_f32(n, BASE_SEED + 2)], [keep_count(n, num, den)],
                    "GPT-2-small post-GELU activation")


def config3() -> Workload:
    n = 32 * 256 * 56 * 56
    return Workload("cfg3_resnet101_grad_32x256x56x56_f32_k1pct", "f32", (32, 256, 56, 56),
                    [student_t_f32(n, BASE_SEED + 3)], [keep_count(n, 1, 100)],
                    "ResNet-101 activation gradient, 1e-3 * t(3)")


def config4(num_segments: int = 24, seg_shape=(8, 1024, 1024)) -> Workload:
    """Segmented batch; keep fraction per segment log-uniform in [0.1 %, 20 %]."""
    n = int(np.prod(seg_shape))
    rho = np.exp(_rng(BASE_SEED + 4).uniform(np.log(1e-3), np.log(0.2), size=num_segments))
    ks = [max(1, int(np.floor(float(n) * float(r)))) for r in rho]
    tensors = [normal_f32(n, BASE_SEED + 4 + 100 * s) for s in range(num_segments)]
    return Workload("cfg4_gpt2m_hidden_%dx8x1024x1024_f32_adaptive" % num_segments, "f32", seg_shape,
                    tensors, ks, "GPT-2-medium hidden activations, per-link adaptive ratios")


def config4_links(num_segments: int = 24, seg_shape=(8, 1024, 1024)) -> Workload:
    """The tensors of config 4, each crossing a link of its own; the keep counts are left to the
    bandwidth-adaptive rule.  Link bandwidths span the range of the paper's testbeds (8 Mbps to
    10 Gbps, abstract and Sec. 7): the two ends are present and the rest is log-uniform between them;
    latencies are log-uniform in 0.1 ms to 50 ms, the slower links tending to the longer ones as for
    links between distant sites.  r = 100 and coefficient 3 as in the paper's experiments."""
    w = config4(num_segments, seg_shape)
    rng = _rng(BASE_SEED + 40)
    lo, hi = 8e6 / 8.0, 10e9 / 8.0  # bytes per second
    bw = np.exp(rng.uniform(np.log(lo), np.log(hi), size=num_segments))
    bw[0], bw[-1] = lo, hi
    order = rng.permutation(num_segments)
    bw = bw[order]
    lat = np.exp(rng.uniform(np.log(1e-4), np.log(5e-2), size=num_segments))
    lat = np.sort(lat)[np.argsort(np.argsort(-bw))]  # longest latency on the lowest bandwidth
    return Workload("cfg4r_gpt2m_hidden_%dx8x1024x1024_f32_planned" % num_segments, "f32", seg_shape, w.tensors, [],
                    "GPT-2-medium hidden activations, keep counts planned from 8 Mbps - 10 Gbps links",
                    alpha=[float(v) for v in lat], beta=[float(1.0 / v) for v in bw], r_user=100.0, coeff=3.0)


def config5() -> Workload:
    n = 16 * 1024 * 1600
    return Workload("cfg5_gpt2xl_hidden_16x1024x1600_bf16_k0.5pct", "bf16", (16, 1024, 1600),
                    [normal_bf16(n, BASE_SEED + 5)], [keep_count(n, 5, 1000)],
                    "GPT-2-XL hidden activation rounded to bf16: many ties at the threshold")


def config5_f16() -> Workload:
    n = 16 * 1024 * 1600
    return Workload("cfg5h_gpt2xl_hidden_16x1024x1600_f16_k0.5pct", "f16", (16, 1024, 1600),
                    [normal_f16(n, BASE_SEED + 5)], [keep_count(n, 5, 1000)],
                    "GPT-2-XL hidden activation rounded to IEEE binary16")


def config_small(num_tensors: int = 128) -> Workload:
    """Many small messages in one call: the launch-bound regime of small models on small inputs
    (the paper's ResNet-18 runs on 3x32x32 images, Sec. 7.1): 1024 to 8192 elements each, k = 1 %."""
    sizes = [8192, 4096, 2048, 1024]  # 512x4x4, 256x4x4, 128x4x4, 64x4x4
    ns = [sizes[i % len(sizes)] for i in range(num_tensors)]
    tensors = [normal_f32(n, BASE_SEED + 6 + 100 * s) for s, n in enumerate(ns)]
    return Workload("small_%dx_1k_to_8k_f32_k1pct" % num_tensors, "f32", (num_tensors,), tensors,
                    [keep_count(n, 1, 100) for n in ns], "many small messages, N(0,1)")


def config_resnet18_samples(num_tensors: int = 64) -> Workload:
    """Per-sample stage outputs of a ResNet-18 on 32x32 inputs (64x32x32, 128x16x16, 256x8x8, 512x4x4),
    many of them in one call, k = 1 %."""
    sizes = [65536, 32768, 16384, 8192]
    ns = [sizes[i % len(sizes)] for i in range(num_tensors)]
    tensors = [normal_f32(n, BASE_SEED + 7 + 100 * s) for s, n in enumerate(ns)]
    return Workload("resnet18_samples_%dx_8k_to_64k_f32_k1pct" % num_tensors, "f32", (num_tensors,), tensors,
                    [keep_count(n, 1, 100) for n in ns], "per-sample ResNet-18 stage outputs, N(0,1)")


def small_case(kind: str, n: int, seed: int, dtype: str = "f32") -> np.ndarray:
    """Small adversarial inputs for parity tests.  ``kind`` picks the value structure."""
    rng = _rng(seed)
    if kind == "normal":
        x = rng.standard_normal(n, dtype=np.float32)
    elif kind == "all_equal":
        x = np.full(n, 1.5, dtype=np.float32)
    elif kind == "all_zero":
        x = np.zeros(n, dtype=np.float32)
    elif kind == "signed_zero_mix":
        x = np.where(rng.random(n) < 0.5, np.float32(0.0), np.float32(-0.0)).astype(np.float32)
    elif kind == "few_levels":  # heavy ties: values from a handful of magnitudes, random signs
        levels = np.array([0.25, 0.5, 1.0, 2.0, 3.0], dtype=np.float32)
        x = levels[rng.integers(0, levels.size, size=n)] * rng.choice(np.array([-1, 1], dtype=np.float32), size=n)
    elif kind == "sparse":  # mostly exact zeros (ReLU-like gradient), a few non-zeros
        x = rng.standard_normal(n, dtype=np.float32)
        x[rng.random(n) < 0.97] = 0.0
    elif kind == "nonfinite":  # finite values with some +-Inf, NaN (two payloads) and denormals
        x = rng.standard_normal(n, dtype=np.float32)
        u = x.view(np.uint32)
        pick = rng.random(n)
        u[pick < 0.01] = 0x7F800000
        u[(pick >= 0.01) & (pick < 0.02)] = 0xFF800000
        u[(pick >= 0.02) & (pick < 0.03)] = 0x7FC00000
        u[(pick >= 0.03) & (pick < 0.04)] = 0xFFC01234
        u[(pick >= 0.04) & (pick < 0.06)] = rng.integers(1, 1 << 22, size=n, dtype=np.uint32)[(pick >= 0.04) & (pick < 0.06)]
    elif kind == "random_bits":  # every bit pattern equally likely
        x = rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32).view(np.float32)
    elif kind == "descending":  # (counted in fp64: an fp32 arange has step 0 once n passes 2^24)
        x = np.arange(n, 0, -1, dtype=np.float64).astype(np.float32)
    elif kind == "ascending":
        x = np.arange(1, n + 1, dtype=np.float64).astype(np.float32)
    else:
        raise ValueError(kind)
    if dtype == "bf16":
        if kind in ("nonfinite", "random_bits"):
            return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
        return f32_to_bf16_bits(x)
    if dtype == "f16":  # IEEE binary16 as numpy float16 (bf16 travels as uint16, so the two stay apart)
        if kind == "random_bits":
            return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16).view(np.float16)
        with np.errstate(over="ignore"):
            h = x.astype(np.float16)  # values past 65504 become Inf: one more tie class
        if kind == "nonfinite":  # fp32 denormals round to 0 in binary16: plant binary16 denormals and NaN payloads
            u = h.view(np.uint16)
            pick = _rng(seed + 1).random(n)
            u[pick < 0.02] = _rng(seed + 2).integers(1, 1 << 10, size=n, dtype=np.uint16)[pick < 0.02]
            u[(pick >= 0.02) & (pick < 0.03)] = 0x7E00
            u[(pick >= 0.03) & (pick < 0.04)] = 0xFD55
        return h
    return x
