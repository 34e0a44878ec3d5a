"""AddressSanitizer + UndefinedBehaviorSanitizer over the host code (CPU only): the oracle's C source
and the library's host-only entry points are compiled from source into one instrumented program
(tests/c/sanitize_host.c) that walks their edge cases with exactly sized heap buffers."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_and_host_entry_points_under_asan_and_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2410_12707_amd", "csrc")]
    objs = []
    for cc, std, src in (("gcc", "-std=c11", os.path.join(ROOT, "oracle", "adatopk_oracle.c")),
                         ("g++", "-std=c++17", os.path.join(ROOT, "paper_2410_12707_amd", "csrc", "adatopk_host.cpp")),
                         ("gcc", "-std=c11", os.path.join(ROOT, "tests", "c", "sanitize_host.c"))):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        subprocess.run([cc, std, "-Wall", "-Wextra", "-Werror"] + san + inc + ["-c", src, "-o", obj], check=True)
        objs.append(obj)
    exe = str(tmp_path / "sanitize_host")
    subprocess.run(["g++"] + san + objs + ["-o", exe, "-lm"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=600, env=env)
    assert r.returncode == 0 and "sanitized host run ok" in r.stdout, (r.returncode, r.stdout[-500:], r.stderr[-3000:])
