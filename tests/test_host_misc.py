"""Host-side checks that need neither a GPU nor the oracle's arithmetic: the benchmark's command
line contract, the seeded input generators, and the product path's refusal to run without its library."""
import json
import os
import subprocess
import sys

import numpy as np

from paper_2410_12707_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                       stderr=subprocess.PIPE, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_workloads_match_the_benchmark_configurations():
    with open(os.path.join(ROOT, "BASELINE.json")) as f:
        base = json.load(f)
    assert "configs" in base and len(base["configs"]) >= 5
    w1 = wl.config1()
    assert w1.tensors[0].size == 4 * 128 * 768 and w1.ks == [3932] and w1.tensors[0].dtype == np.float32
    assert wl.keep_count(25_165_824, 1, 100) == 251_658 and wl.keep_count(26_214_400, 5, 1000) == 131_072
    s = wl.config_small()
    assert len(s.tensors) == 128 and max(t.size for t in s.tensors) == 8192 and all(k == t.size // 100 for k, t in zip(s.ks, s.tensors))
    r = wl.config_resnet18_samples()
    assert sorted({t.size for t in r.tensors}) == [8192, 16384, 32768, 65536]


def test_generators_are_seeded_and_typed():
    a, b = wl.normal_f32(1000, 5), wl.normal_f32(1000, 5)
    assert np.array_equal(a, b) and not np.array_equal(a, wl.normal_f32(1000, 6))
    h = wl.normal_bf16(1000, 5)
    assert h.dtype == np.uint16
    back = wl.bf16_bits_to_f32(h)
    assert np.all(np.abs(back - a) <= np.abs(a) * 2.0 ** -8)  # round to nearest: half an ulp of 8 significand bits
    assert wl.normal_f16(1000, 5).dtype == np.float16
    for kind in ("normal", "all_equal", "all_zero", "signed_zero_mix", "few_levels", "sparse", "nonfinite", "random_bits",
                 "descending", "ascending"):
        for dtype, npdt in (("f32", np.float32), ("bf16", np.uint16), ("f16", np.float16)):
            x = wl.small_case(kind, 257, seed=3, dtype=dtype)
            assert x.dtype == npdt and x.size == 257
            assert np.array_equal(x.view(np.uint8), wl.small_case(kind, 257, seed=3, dtype=dtype).view(np.uint8))
    g = wl.gelu_of_normal_f32(100_000, 1)
    assert g.min() > -0.2 and (g < 0).mean() > 0.4  # GELU: negative half squashed into (-0.17, 0)


def test_binding_fails_loudly_without_the_library(tmp_path):
    code = ("import os, sys; sys.path.insert(0, %r); os.environ['ADATOPK_LIBRARY'] = %r\n"
            "from paper_2410_12707_amd import binding as B\n"
            "try:\n    B.load_library()\nexcept Exception as e:\n    print('RAISED', type(e).__name__); sys.exit(0)\n"
            "sys.exit(3)\n") % (ROOT, str(tmp_path / "missing.so"))
    r = subprocess.run([sys.executable, "-c", code], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)
    assert r.returncode == 0 and "RAISED" in r.stdout, (r.stdout, r.stderr)
