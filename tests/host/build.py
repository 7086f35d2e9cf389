"""Builds tests/host/abi_standalone: the C ABI driven from a plain HIP program
(no Python, no PyTorch), linked against the in-tree libkt.so and the CPU
checker's libkt_oracle.so.  Test infrastructure."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
EXE = os.path.join(HERE, "abi_standalone")


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = EXE + ".tmp%d" % os.getpid()
    cmd = [hipcc, "-O2", "-std=c++17", "--offload-arch=gfx950", "-I", os.path.join(ROOT, "include"),
           os.path.join(HERE, "abi_standalone.cpp"), "-o", tmp,
           "-L", os.path.join(ROOT, "paper_2505_10183_amd"), "-lkt", "-L", os.path.join(ROOT, "oracle"), "-lkt_oracle",
           "-Wl,-rpath,$ORIGIN/../../paper_2505_10183_amd", "-Wl,-rpath,$ORIGIN/../../oracle"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, EXE)
    return EXE


if __name__ == "__main__":
    print(build(verbose=True))
