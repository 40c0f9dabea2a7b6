"""Compile the HIP sources under csrc/ into libcsr_hip.so (gfx950 only), next to this file.

hipcc cross-compiles without a GPU.  The library leaves the HIP runtime to whoever loads it
(PyTorch's own copy once torch is imported), so it must be loaded after `import torch`.
"""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libcsr_hip.so")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


# decode.hip: the streaming kernel's rounds are unrolled by pragma (the scores of a thread's tokens live in registers);
# the 32 rounds of its four-head variant exceed the compiler's default size limit for such an unroll, and a loop left
# rolled would put the score array into scratch memory.
PER_FILE_FLAGS = {"decode.hip": ["-mllvm", "-pragma-unroll-threshold=200000"]}


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False, extra=()) -> str:
    """One hipcc compile per source file, side by side, then one link."""
    import concurrent.futures
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    compile_flags = [f for f in FLAGS if f != "-shared"]
    with tempfile.TemporaryDirectory(prefix="csr_build_") as tmp:
        def compile_one(src):
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            cmd = [hipcc, *compile_flags, *PER_FILE_FLAGS.get(os.path.basename(src), []), *extra, "-I", INCLUDE, "-I", CSRC, "-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj
        with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
            objs = list(pool.map(compile_one, sources()))
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", *objs, "-o", LIB + ".tmp"]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


C_SMOKE_SRC = os.path.join(os.path.dirname(HERE), "tests", "c_abi", "smoke.c")
C_SMOKE_BIN = os.path.join(HERE, "csr_c_smoke.bin")


def build_c_smoke(verbose: bool = False) -> str:
    """The plain-C user of the ABI (tests/c_abi/smoke.c), compiled by the host C compiler against the library."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = [os.environ.get("CC", "gcc"), "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", INCLUDE,
           "-I", os.path.join(rocm, "include"), C_SMOKE_SRC, "-o", C_SMOKE_BIN, "-L", HERE, "-lcsr_hip",
           "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return C_SMOKE_BIN


PROBE_SRC = os.path.join(CSRC, "probe", "mfma_rate.hip")
PROBE_BIN = os.path.join(HERE, "mfma_rate.bin")


def build_probe(verbose: bool = False) -> str:
    """The stand-alone matrix-core rate probe (csrc/probe/mfma_rate.hip): what the chip sustains on MFMA alone."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           PROBE_SRC, "-o", PROBE_BIN]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return PROBE_BIN


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
    print(build_c_smoke(verbose=True))
    print(build_probe(verbose=True))
