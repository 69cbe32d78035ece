"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only).

oracle/sanitize_check.c calls every exported layer function on exact-size heap buffers over shapes that
reach the edges of the index arithmetic; built with -fsanitize=address,undefined as a program of its own
(the sanitizer runtime linked statically, so nothing has to be preloaded) any access past a buffer or
undefined arithmetic ends it with a non-zero status.
"""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_check")
    src = os.path.join(ROOT, "oracle", "sanitize_check.c")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
                           "-o", exe, src, "-lm"], cwd=os.path.join(ROOT, "oracle"))
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120,
                       env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", OMP_NUM_THREADS="4"))
    assert r.returncode == 0, (r.stdout[-500:], r.stderr[-3000:])
    assert "sanitize_check ok" in r.stdout and "runtime error" not in r.stderr
