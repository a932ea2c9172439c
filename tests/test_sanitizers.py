"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

The planner (csrc/plan.cpp, no HIP call in it) and the C oracle are compiled with the host
compiler and -fsanitize=address,undefined, each with a small driver from tests/sanitize/:
the planner runs over the random batches of test_plan_random_batches (and re-plans each
with grown lengths), the oracle over the two-token worked example and a small paged fp8
problem.  Any report makes the program exit non-zero.  The sanitizer runtime is linked
statically so that it does not depend on the order of preloaded libraries.
"""
import os
import random
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", OMP_NUM_THREADS="2")


def _build(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0 and "static-libasan" in res.stderr:
        pytest.skip("host compiler has no static sanitizer runtime")
    assert res.returncode == 0, res.stderr[-2000:]


def test_planner_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "plan_san")
    _build(["g++", "-std=c++17", *SAN, os.path.join(ROOT, "tests", "sanitize", "plan_driver.cpp"),
            os.path.join(ROOT, "paper_2511_22481_amd", "csrc", "plan.cpp"), "-o", exe])
    rng = random.Random(7)          # the batches of test_plan_random_batches
    lines = []
    for _ in range(60):
        B = rng.randint(1, 9)
        lens = [rng.choice([0, 1, rng.randint(1, 5000)]) for _ in range(B)]
        S = rng.choice([0, 5, 64, 128, 1000])
        W = rng.choice([0, 7, 512, 2048, 9000])
        H = rng.choice([1, 16, 48, 128, 160])
        hint = rng.choice([0, 0, 1, 2, 3, 7, 1000])
        cus = rng.choice([1, 8, 256])
        lines.append(" ".join(map(str, [B, H, S, W, hint, 0, cus] + lens)))
    # the benchmark shapes and several queries per sequence
    lines.append(" ".join(map(str, [64, 128, 128, 2048, 0, 0, 256] + [32768] * 64)))
    lines.append(" ".join(map(str, [32, 128, 128, 8192, 0, 0, 256] + [131072] * 32)))
    lines.append(" ".join(map(str, [3, 16, 64, 100, 2, 3, 8] + [3, 500, 129])))
    res = subprocess.run([exe], input="\n".join(lines) + "\n", capture_output=True, text=True, env=ENV)
    assert res.returncode == 0, (res.stdout[-500:], res.stderr[-3000:])
    assert res.stdout.strip() == f"ok {len(lines)}"


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _build(["gcc", "-std=c11", *SAN, "-fopenmp", os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
            os.path.join(ROOT, "oracle", "omniattn_oracle.c"), "-o", exe, "-lm"])
    res = subprocess.run([exe], capture_output=True, text=True, env=ENV)
    assert res.returncode == 0, (res.stdout[-500:], res.stderr[-3000:])
    assert res.stdout.strip() == "ok"
