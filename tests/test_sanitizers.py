"""The oracle and the host side of the library under AddressSanitizer + UBSan (CPU only).

Each is built a second time with the sanitizers into a temporary directory and exercised in a
child process that preloads the matching sanitizer runtime: the oracle (gcc) on the hand-worked
fixtures, the pins and a set of tiny random searches in every mode; the library's host code
(hipcc, host side only) on the validation and staging paths that run without a GPU.  A report
from either sanitizer ends the child with a non-zero status.
"""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _first(patterns):
    for p in patterns:
        hit = sorted(glob.glob(p))
        if hit:
            return hit[-1]
    return None


GCC_ASAN = _first(["/usr/lib/gcc/x86_64-linux-gnu/*/libasan.so"])
CLANG_ASAN = _first(["/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so",
                     "/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"])


def _child(env_extra, args, timeout):
    env = dict(os.environ)
    env.update(env_extra)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    out = subprocess.run([sys.executable] + args, cwd=ROOT, env=env, capture_output=True, text=True, timeout=timeout)
    tail = (out.stdout + out.stderr)[-4000:]
    assert out.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    return out.stdout


ORACLE_EXERCISE = r"""
import sys
sys.path.insert(0, "tests")
import numpy as np
import oracle
from paper_2603_08797_amd import workloads as W
n = 0
for seed in range(20):
    pb, se = W.tiny_random(seed)
    o = oracle.Oracle.from_problem(pb)
    for cap in (0, se.prune_cap or 2 * pb.V):
        res, bl, md = o.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, cap, threads=2)
        for D in se.demand_mrps.tolist():
            K, space, tr = o.space(D, se.slo_latency_us, cap)
            if space:
                o.eval(D, se.slo_latency_us, se.slo_accuracy, cap, np.arange(min(space, 64), dtype=np.uint64))
                o.search_range(D, se.slo_latency_us, se.slo_accuracy, cap, 0, space, threads=2)
            for t in range(pb.T):
                o.pruned(D, se.slo_latency_us, cap, t)
        n += len(res)
    o.accuracy_margin(se.slo_accuracy)
    o.set_objective(1, 1.0, 0.035)
    o.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0, threads=2)
    o.objective_margin(int(se.demand_mrps[0]), se.slo_latency_us, se.slo_accuracy, 0)
    o.set_objective(0, 1.0, 0.035)
    for a, s, t in ((0, 1, 1), (1, 0, 1), (1, 1, 0), (0, 0, 0)):
        o.set_search_space(a, s, t)
        o.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0, threads=1)
        o.budget_margin()
    o.close()
for seed in range(8):
    pb, se = W.tiny_mixture(3000 + seed)
    if pb.capacity_units == 0:
        import dataclasses
        pb = dataclasses.replace(pb, capacity_units=30)
    o = oracle.Oracle.from_problem(pb)
    o.set_mixtures(True)
    for cap in (4, 12, 400):
        o.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, cap, threads=2)
        o.options(int(se.demand_mrps[0]), se.slo_latency_us, cap, 0)
        o.mixture_margin(int(se.demand_mrps[0]), se.slo_latency_us, se.slo_accuracy, cap)
    o.close()
for seed in range(6):
    pb, se = W.tiny_random(700 + seed, T=3)
    if pb.E == 0:
        continue
    o = oracle.Oracle.from_problem(pb)
    o.set_factors(W.random_factors(pb, seed))
    o.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap, threads=2)
    o.close()
print("oracle exercised:", n, "levels")
"""


@pytest.mark.skipif(GCC_ASAN is None, reason="gcc's libasan.so not found")
def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    lib = str(tmp_path / "libjsv_oracle_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-fno-omit-frame-pointer", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
                           "-o", lib, os.path.join(ROOT, "oracle", "jsv_oracle.c")])
    with open(lib, "rb") as f:
        assert b"__asan_init" in f.read()                 # the instrumentation is really there
    env = {"JSV_ORACLE_LIBRARY": lib, "LD_PRELOAD": GCC_ASAN}
    out = _child(env, ["-c", ORACLE_EXERCISE], 600)
    assert "oracle exercised" in out
    # the hand-worked fixtures and the pins, unchanged, against the instrumented build
    _child(env, ["-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_oracle_golden.py",
                 "tests/test_oracle_pins.py"], 600)


@pytest.mark.skipif(CLANG_ASAN is None, reason="clang's asan runtime not found")
def test_library_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    from paper_2603_08797_amd import build as hip_build
    lib = str(tmp_path / "libjsv_san.so")
    srcs = [os.path.join(hip_build.CSRC, s) for s in hip_build.SOURCES]
    flags = [f for f in hip_build.FLAGS if f != "-O3"]
    subprocess.check_call([os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")] + flags +
                          ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                           "-Xarch_host", "-fno-sanitize-recover=undefined", "-x", "hip"] + srcs +
                          ["-shared", "-o", lib], stderr=subprocess.DEVNULL)
    with open(lib, "rb") as f:
        assert b"__asan_init" in f.read()
    env = {"JSV_LIBRARY": lib, "LD_PRELOAD": CLANG_ASAN}
    # validation, staging (topological order, shares, A_max, budgets), batch staging, the size
    # check of the static-scratch entry point: everything that runs before the first device call
    _child(env, ["-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_host_abi.py"], 600)
