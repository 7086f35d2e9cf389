"""Builds libkt.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkt.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 instructions are switched off for all device code
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
COMMON = ["-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-ffp-contract=off", "-Wall", "-Wextra",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(verbose: bool = False, extra_defines=(), out: str = LIB) -> str:
    """Compile and link the library.  `extra_defines` are passed to every
    compile (-DKT_TILE_BYTES=8192, -DKT_NT_LOAD=0, -DKT_NT_STORE=0,
    -DKT_LDS_TENSORS=1 build the variants used to compare design choices);
    `out` names the shared library to write (default: the in-tree libkt.so)."""
    objs = []
    tag = "" if out == LIB else ".variant%d" % os.getpid()
    for name in ("kt_plan.cpp", "kt_sampler.cpp", "kt_api.cpp", "kt_pack_unpack.hip", "kt_reduce.hip",
                 "kt_fused.hip", "kt_sgd.hip", "kt_fused_sgd.hip", "kt_static.hip"):
        src = os.path.join(CSRC, name)
        obj = os.path.join(CSRC, os.path.splitext(name)[0] + tag + ".o")
        cmd = [HIPCC] + COMMON + list(extra_defines)
        if name.endswith(".hip"):
            cmd += DEVICE_FLAGS
        cmd += ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        objs.append(obj)
    tmp = out + ".tmp%d" % os.getpid()
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, out)
    if tag:
        for o in objs:
            os.remove(o)
    return out


PROBE_SRC = os.path.join(ROOT, "bench_probe.hip")
PROBE_LIB = os.path.join(ROOT, "libkt_bench_probe.so")


def build_bench_probe(verbose: bool = False) -> str:
    """Compile the benchmark's read-only bandwidth probe (bench_probe.hip beside
    bench.py) into its own small shared library; the C-ABI library does not
    contain it."""
    tmp = PROBE_LIB + ".tmp%d" % os.getpid()
    cmd = [HIPCC, "-O3", "-std=c++17", "-fPIC", "-shared"] + DEVICE_FLAGS + [PROBE_SRC, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, PROBE_LIB)
    return PROBE_LIB


if __name__ == "__main__":
    args = sys.argv[1:]
    target = LIB
    if "--out" in args:
        i = args.index("--out")
        target = os.path.abspath(args[i + 1])
        del args[i:i + 2]
    print(build(verbose=True, extra_defines=args, out=target))
    if target == LIB:
        print(build_bench_probe(verbose=True))
