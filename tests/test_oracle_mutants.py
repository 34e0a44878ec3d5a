"""The pins must be able to fail: every planted mistake below, applied to a COPY of the oracle's
source on the CPU, has to make the pin suite fail.  A mistake that survives means the oracle could
carry it unnoticed, and every parity claim built on the oracle with it.

Each case edits one expression of `oracle/adatopk_oracle.c` or `oracle/wire_format.py` in a
temporary copy of the tree, rebuilds it there, and runs the pin tests of that copy in a subprocess.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

C = "oracle/adatopk_oracle.c"
W = "oracle/wire_format.py"
PINS = "tests/test_oracle_pins.py"
WIRE = "tests/test_wire_format.py"

# (name, file, text to replace (must occur; `nth` picks which occurrence), replacement, test file run)
MUTANTS = [
    ("ties_to_highest_index", C, "if (a->idx != b->idx) return (a->idx < b->idx) ? -1 : 1;",
     "if (a->idx != b->idx) return (a->idx < b->idx) ? 1 : -1;", 0, PINS),
    ("smallest_keys_first", C, "if (a->key != b->key) return (a->key > b->key) ? -1 : 1;",
     "if (a->key != b->key) return (a->key > b->key) ? 1 : -1;", 0, PINS),
    ("sign_kept_in_fp32_key", C, "keys[i] = u & 0x7FFFFFFFu;", "keys[i] = u;", 0, PINS),
    ("sign_kept_in_bf16_key", C, "keys[i] = (uint32_t)(x[i] & 0x7FFFu);", "keys[i] = (uint32_t)x[i];", 0, PINS),
    ("sign_kept_in_fp16_key", C, "keys[i] = (uint32_t)(x[i] & 0x7FFFu);", "keys[i] = (uint32_t)x[i];", 1, PINS),
    ("error_over_all_elements", C, "if (!sel[i]) s += (double)x[i] * (double)x[i];",
     "s += (double)x[i] * (double)x[i];", 0, PINS),
    ("error_without_square_root", C, "*err = (float)sqrt(s);", "*err = (float)s;", 0, PINS),
    ("zero_fill_one_short", C, "memset(y, 0, (size_t)n * sizeof *y);",
     "memset(y, 0, (size_t)(n > 0 ? n - 1 : 0) * sizeof *y);", 0, PINS),
    ("output_not_resorted_by_index", C, "qsort(idx, (size_t)k, sizeof *idx, cmp_idx_asc);", "", 0, PINS),
    ("ratio_rule_inverted", C, "double v = coeff * r * R[i] / Rmax;", "double v = coeff * r * Rmax / (R[i] > 0 ? R[i] : 1);",
     0, PINS),
    ("ratio_rule_without_floor_of_one", C, "r_out[i] = v > 1.0 ? v : 1.0;", "r_out[i] = v;", 0, PINS),
    ("keep_count_rounded_up", C, "double q = floor((double)n / r_i);", "double q = ceil((double)n / r_i);", 0, PINS),
    ("pipeline_counts_every_micro_batch", C, "return sum + (double)(n_b - 1) * worst;",
     "return sum + (double)n_b * worst;", 0, PINS),
    ("compressed_pipeline_variants_swapped", C, "if (variant == 0) return sum + coeff", "if (variant != 0) return sum + coeff",
     0, PINS),
    ("fp16_exponent_bias_off_by_one", C, "else v = ldexp((double)(1024 + m), e - 25);",
     "else v = ldexp((double)(1024 + m), e - 24);", 0, PINS),
    ("fp16_denormals_flushed", C, "if (e == 0) v = ldexp((double)m, -24);", "if (e == 0) v = 0.0;", 0, PINS),
    ("rounding_truncates", C, "double r = rint(s / quantum) * quantum;", "double r = trunc(s / quantum) * quantum;", 0, PINS),
    ("bf16_one_significand_bit_short", C, "round_to_format(s, 8, -126, 127)", "round_to_format(s, 7, -126, 127)", 0, PINS),
    ("accumulate_overwrites", C, "y[idx[j]] = (float)((double)y[idx[j]] + (double)val[j]);",
     "y[idx[j]] = val[j];", 0, PINS),
    ("segmented_bf16_values_at_previous_tensors_offset", C,
     "int rc = oracle_compress_bf16(x + in_offset[s], in_offset[s + 1] - in_offset[s], k[s],\n"
     "                                      idx + out_offset[s], val + out_offset[s], err ? err + s : NULL);",
     "int rc = oracle_compress_bf16(x + in_offset[s], in_offset[s + 1] - in_offset[s], k[s],\n"
     "                                      idx + out_offset[s], val + out_offset[s > 0 ? s - 1 : s], err ? err + s : NULL);", 0, PINS),
    ("segmented_f16_reads_neighbours_k", C,
     "int rc = oracle_compress_f16(x + in_offset[s], in_offset[s + 1] - in_offset[s], k[s],",
     "int rc = oracle_compress_f16(x + in_offset[s], in_offset[s + 1] - in_offset[s], k[s > 0 ? s - 1 : s],", 0, PINS),
    ("segmented_f32_error_of_first_tensor_only", C,
     "idx + out_offset[s], val + out_offset[s], err ? err + s : NULL);",
     "idx + out_offset[s], val + out_offset[s], err ? err : NULL);", 0, PINS),
    ("segmented_bf16_tensor_length_from_k", C,
     "int rc = oracle_compress_bf16(x + in_offset[s], in_offset[s + 1] - in_offset[s], k[s],",
     "int rc = oracle_compress_bf16(x + in_offset[s], in_offset[s + 1] - in_offset[s] - (s == 5), k[s],", 0, PINS),
    ("wire_padding_to_8", W, "return HEADER_BYTES + (k * index_bytes + 15) // 16 * 16",
     "return HEADER_BYTES + (k * index_bytes + 7) // 8 * 8", 0, WIRE),
    ("wire_big_endian_indices", W, 'dtype="<i4" if index_bytes == 4 else "<i8").tobytes()',
     'dtype=">i4" if index_bytes == 4 else ">i8").tobytes()', 0, WIRE),
    ("wire_n_and_k_swapped", W, "index_bytes, float(err_norm), int(n), k,", "index_bytes, float(err_norm), k, int(n),", 0, WIRE),
]


def _copy_tree(dst):
    os.makedirs(os.path.join(dst, "oracle"))
    for f in ("__init__.py", "adatopk_oracle.py", "adatopk_oracle.c", "wire_format.py"):
        shutil.copy(os.path.join(ROOT, "oracle", f), os.path.join(dst, "oracle", f))
    os.makedirs(os.path.join(dst, "tests"))
    for f in ("conftest.py", "test_oracle_pins.py", "test_wire_format.py"):
        shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(dst, "tests", f))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(dst, "tests", "golden"))
    shutil.copytree(os.path.join(ROOT, "paper_2410_12707_amd"), os.path.join(dst, "paper_2410_12707_amd"),
                    ignore=shutil.ignore_patterns("csrc", "__pycache__"))


def _run(dst, test_file):
    env = dict(os.environ, PYTHONPATH=dst, PYTHONDONTWRITEBYTECODE="1")
    return subprocess.run([sys.executable, "-m", "pytest", test_file, "-x", "-q", "-p", "no:cacheprovider"], cwd=dst,
                          env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)


def _replace_nth(text, old, new, nth):
    pos = -1
    for _ in range(nth + 1):
        pos = text.find(old, pos + 1)
        assert pos >= 0, "mutation anchor not found (the oracle changed: update the mutant): %r" % old
    return text[:pos] + new + text[pos + len(old):]


def test_unmutated_copy_passes(tmp_path):
    dst = str(tmp_path / "clean")
    _copy_tree(dst)
    for test_file in (PINS, WIRE):
        r = _run(dst, test_file)
        assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,path,old,new,nth,test_file", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, path, old, new, nth, test_file):
    dst = str(tmp_path / name)
    _copy_tree(dst)
    target = os.path.join(dst, path)
    with open(target) as f:
        text = f.read()
    with open(target, "w") as f:
        f.write(_replace_nth(text, old, new, nth))
    r = _run(dst, test_file)
    assert r.returncode != 0, "no pin noticed the planted mistake '%s'" % name
    assert " failed" in r.stdout or " error" in r.stdout, r.stdout[-2000:]
