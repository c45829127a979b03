"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

The oracle allocates per (sequence, kv head) and indexes through a block table; this builds it
with gcc's sanitizers into a small C program (tests/oracle_sanitize_driver.c) that runs ragged
paged batches in both dtypes, row ranges and spans that reach outside the chunk, the row-subset
mode, the bad-block-id error path and both steering functions, and checks the results against
closed forms.  Any out-of-bounds access, use after free or undefined operation aborts the run."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-Wall", "-Wextra", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-static-libasan", "-static-libubsan",
           os.path.join(ROOT, "tests", "oracle_sanitize_driver.c"), os.path.join(ROOT, "oracle", "hook_oracle.c"),
           "-o", exe, "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert res.stdout.strip().endswith("ok")
