"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): the
oracle source is compiled together with a small C driver that calls every entry point at bucket
sizes 32, 96 and 8192, n = 1, a bucket less one, a whole bucket and a ragged tail, code widths 1, 3
and 8, with one and with three threads (the per-thread bucket arrays live on the OpenMP stacks).
Any report makes the run fail."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-static-libasan", "-static-libubsan",
           "-I", os.path.join(ROOT, "oracle"), os.path.join(ROOT, "oracle", "qsdp_ref.c"),
           os.path.join(ROOT, "tests", "oracle_sanitizer_driver.c"), "-o", exe, "-lm"]
    subprocess.run(cmd, check=True, cwd=ROOT)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="3")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
    assert r.stdout.startswith("done ") and int(r.stdout.split()[1]) > 2000
