"""Build libsignsgd.so (the C-ABI HIP library) for gfx950, in-tree.

    python -m paper_1802_04434_amd.build

Flags: FP contraction off (momentum must round each product and the sum
separately), packed-fp32 instructions disabled, no fast-math.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsignsgd.so")
SOURCES = ["api.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(out=LIB, verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = out + ".tmp%d" % os.getpid()
    cmd = [hipcc, *HIPCC_FLAGS, "-o", tmp] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, out)
    return out


ABI_CHECK = os.path.join(HERE, "abi_check")


def build_abi_check(verbose=False):
    """The stand-alone C++ host program that drives the library without Python
    (csrc/abi_check.cpp); it finds libsignsgd.so next to itself."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    tmp = ABI_CHECK + ".tmp%d" % os.getpid()
    # plain host C++: only the HIP runtime API (hipMalloc, hipMemcpy, streams) and the library
    cmd = ["g++", "-O2", "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(rocm, "include"),
           os.path.join(CSRC, "abi_check.cpp"), "-o", tmp, "-L" + HERE, "-lsignsgd",
           "-L" + os.path.join(rocm, "lib"), "-lamdhip64", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, ABI_CHECK)
    return ABI_CHECK


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_abi_check(verbose=True))
