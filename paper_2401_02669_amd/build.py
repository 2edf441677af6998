"""Build libdistattn.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdistattn.so")
PROBE_LIB = os.path.join(HERE, "libdistattn_probe.so")  # measurement probes (include/distattn_probe.h), bench-only
PROBE_SOURCES = ["read_probe.hip"]
SOURCES = ["distattn_api.hip", "micro_attention_valu.hip", "micro_attention_mfma.hip", "micro_attention_mfma_tiles.hip", "micro_attention_mfma_f32.hip", "combine.hip", "append.hip", "move.hip", "block_pool.cpp", "schedule.cpp", "placement.cpp"]
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-fno-gpu-rdc",
    # packed-fp32 instructions are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-pragmas",
]


C_DRIVER = os.path.join(HERE, "c_abi_driver")


def build_c_driver(verbose=False):
    """The plain-C user of the library (tests/c_abi_driver.c), linked against libdistattn.so and the HIP runtime."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-O1", "-Wall", os.path.join(os.path.dirname(HERE), "tests", "c_abi_driver.c"),
           "-I" + os.path.join(rocm, "include"), "-L" + HERE, "-ldistattn", "-L" + os.path.join(rocm, "lib"), "-lamdhip64",
           "-lm", "-Wl,-rpath," + HERE, "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", C_DRIVER]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return C_DRIVER


def build(verbose=False, extra=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + list(extra)
    for s in SOURCES:
        path = os.path.join(CSRC, s)
        cmd += (["-x", "hip", path] if s.endswith(".cpp") else [path])
    cmd += ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    cmd = [hipcc] + FLAGS + list(extra) + [os.path.join(CSRC, x) for x in PROBE_SOURCES] + ["-o", PROBE_LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    build_c_driver(verbose)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
