"""The library's host-only code under AddressSanitizer and UBSan (CPU build with g++, no GPU, no HIP runtime).

csrc/trace_sim.hip (moe_trace_misses: offline LRU / farthest-next-use analysis of a selection trace) includes
nothing but the public header and the standard library, so it compiles as plain C++.  The sanitizer build is fed
random traces with exact-size heap buffers; its results must equal those of the shipped library, and the sanitizers
must stay silent."""
import os
import shutil
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cases(seed, n):
    r = np.random.default_rng(seed)
    for _ in range(n):
        N = int(r.integers(1, 14))
        K = int(r.integers(1, min(4, N) + 1))
        T = int(r.integers(0, 30))
        policy = int(r.integers(0, 2))
        C_ = int(r.integers(K if policy == 1 else 1, N + 1))
        n_init = int(r.integers(0, C_ + 1))
        init = r.permutation(N)[:n_init].astype(np.int32)
        trace = np.array([r.permutation(N)[:K] for _ in range(T)], np.int32).reshape(T, K)
        yield T, K, N, C_, policy, init, trace


def test_trace_simulator_under_asan_ubsan(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    from paper_2412_00099_amd import binding as B

    exe = tmp_path / "trace_sim_san"
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           "-I", os.path.join(ROOT, "include"),
           "-x", "c++", os.path.join(ROOT, "paper_2412_00099_amd", "csrc", "trace_sim.hip"),
           os.path.join(ROOT, "tests", "host", "trace_sim_driver.cpp"), "-o", str(exe)]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    cases = list(_cases(2024, 400))
    lines = [str(len(cases))]
    for T, K, N, C_, policy, init, trace in cases:
        lines.append(f"{T} {K} {N} {C_} {policy} {len(init)}")
        lines.append(" ".join(map(str, init.tolist())))
        lines.append(" ".join(map(str, trace.ravel().tolist())))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([str(exe)], input="\n".join(lines) + "\n", capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stderr[-2000:]
    assert "ERROR" not in run.stderr and "runtime error" not in run.stderr, run.stderr[-2000:]
    out = run.stdout.strip().splitlines()
    assert out[-1] == "errors 0" and len(out) == len(cases) + 1
    for (T, K, N, C_, policy, init, trace), line in zip(cases, out):
        rc, m, life, ev = map(int, line.split())
        assert rc == B.MOE_OK
        assert (m, life, ev) == B.moe_trace_misses(trace.reshape(T, K), N, C_, policy, init.tolist())
