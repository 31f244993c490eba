"""Builds libjsv.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libjsv.so")
SOURCES = ["jsv_kernels.hip", "jsv_host.cpp"]
HEADERS = ["jsv_device.h", "jsv_launch.h", os.path.join("..", "..", "include", "jsv.h")]
# -packed-fp32-ops off: the compiler must not form packed fp32 instructions
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
         # the hot loops name scalar registers in inline asm: a build in which the compiler has
         # reserved one of them for itself (it then warns) must not come out
         "-Werror=inline-asm"]


PROBE_LIB = os.path.join(HERE, "libjsv_probe.so")
PROBE_SRC = os.path.join(CSRC, "peak_probe.hip")


def build_probe(force: bool = True) -> str:
    """The VALU peak microbenchmark of bench.py --peak-probe: a library of its own."""
    if not force and os.path.exists(PROBE_LIB) and os.path.getmtime(PROBE_LIB) >= os.path.getmtime(PROBE_SRC):
        return PROBE_LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc] + FLAGS + ["-x", "hip", PROBE_SRC, "-shared", "-o", PROBE_LIB])
    return PROBE_LIB


def build(force: bool = True) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    deps = srcs + [os.path.join(CSRC, h) for h in HEADERS]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-Rpass-analysis=kernel-resource-usage", "-x", "hip"] + srcs + ["-shared", "-o", LIB]
    done = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    remarks = [l for l in done.stderr.splitlines() if "-Rpass-analysis=kernel-resource-usage" in l]
    if done.returncode != 0 or " warning: " in done.stderr:
        print("\n".join(l for l in done.stderr.splitlines() if l not in remarks and "packed-fp32-ops" not in l))
    if done.returncode != 0:
        raise subprocess.CalledProcessError(done.returncode, cmd)
    # The enumeration kernels may not spill vector registers to scratch memory: the inline asm of
    # their hot loops names scalar registers by number, and in a build with scratch in it the
    # compiler keeps state of its own in registers that it then reserves.
    name = ""
    for l in remarks:
        if "Function Name:" in l:
            name = l.split("Function Name:")[1].split()[0]
        elif ("enumerate_kernel" in name and "ScratchSize [bytes/lane]:" in l
              and int(l.split("ScratchSize [bytes/lane]:")[1].split()[0]) != 0):
            os.remove(LIB)
            raise RuntimeError(f"kernel {name} uses scratch memory; lower its register pressure")
    return LIB


if __name__ == "__main__":
    print(build())
    print(build_probe())
