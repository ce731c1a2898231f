"""Builds libbms.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbms.so")

OBJ_DIR = os.path.join(HERE, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_lib(verbose: bool = False, incremental: bool = False) -> str:
    """Compile every HIP source into paper_2311_02909_amd/libbms.so: one object per source (compiled side by
    side), then one link.  Always recompiles everything unless `incremental` (then only sources newer than their
    object, or everything when a header changed)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    include = os.path.join(os.path.dirname(HERE), "include")
    os.makedirs(OBJ_DIR, exist_ok=True)
    headers = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(include, "*.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            return obj
        cmd = [hipcc] + HIPCC_FLAGS + ["-I", include, "-c", "-o", obj, src]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        objs = list(pool.map(compile_one, sources()))
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", tmp] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


PROBE_SRC = os.path.join(HERE, "csrc_probe", "probes.hip")
PROBE_LIB = os.path.join(HERE, "libbms_probe.so")


def build_probes(verbose: bool = False) -> str:
    """The rate probes of bench.py (--line-probe, --lds-probe): a library of their own, paper_2311_02909_amd/libbms_probe.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = PROBE_LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + ["-shared", "-o", tmp, PROBE_SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, PROBE_LIB)
    return PROBE_LIB


C_CLIENT_SRC = os.path.join(os.path.dirname(HERE), "tests", "c_abi", "bms_c_client.c")
C_CLIENT = os.path.join(os.path.dirname(HERE), "tests", "c_abi", "bms_c_client")


def build_c_client(verbose: bool = False) -> str:
    """The plain-C client of the library used by tests/test_gpu_c_abi.py (gcc, C99; links libbms.so and the HIP runtime)."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
           "-I", os.path.join(os.path.dirname(HERE), "include"), "-o", C_CLIENT, C_CLIENT_SRC,
           "-L", HERE, "-lbms", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_2311_02909_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return C_CLIENT


if __name__ == "__main__":
    import sys
    print(build_lib(verbose=True, incremental="--incremental" in sys.argv))
    print(build_probes(verbose=True))
    print(build_c_client(verbose=True))
