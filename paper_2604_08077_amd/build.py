"""Build ``libadaspark.so`` (HIP, gfx950 only) in-tree with hipcc.

``python -m paper_2604_08077_amd.build`` or ``build()`` compiles every source
under ``csrc/`` each time it is called; ``lib_path()`` just names the result.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libadaspark.so")
OBJ_DIR = os.path.join(_HERE, "_build")

SOURCES = ["api.hip", "pool.hip", "select.hip", "kvpack.hip", "attn_compact.hip", "attn_walk.hip", "attn_pairs.hip", "ffn.hip",
           "ffn_gemm.hip", "attn_bwd.hip", "probe.hip"]
HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-Wall",
    "-Wno-unused-result",
    "-Wno-inline-asm",
    # packed-fp32 instruction selection is switched off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def lib_path() -> str:
    return LIB


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = False, extra_flags=()) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
        warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if verbose and warn:
            print(warn, flush=True)
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    tmp = LIB + f".tmp{os.getpid()}"
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    return LIB


C_CLIENT_SRC = os.path.join(os.path.dirname(_HERE), "tests", "c_client", "abi_client.c")
C_CLIENT = os.path.join(os.path.dirname(_HERE), "tests", "c_client", "abi_client")


def build_c_client() -> str:
    """The plain-C client of the C ABI (tests/c_client/abi_client.c): gcc in C99 mode, linked against the built
    library and the HIP runtime; tests/test_gpu_c_client.py runs it on the GPU machine."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    include = os.path.join(os.path.dirname(_HERE), "include")
    tmp = C_CLIENT + f".tmp{os.getpid()}"
    subprocess.check_call(["gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I" + include,
                           "-I" + os.path.join(rocm, "include"), C_CLIENT_SRC, "-o", tmp, "-L" + _HERE, "-ladaspark",
                           "-L" + os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
                           "-Wl,-rpath,$ORIGIN/../../paper_2604_08077_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")])
    os.replace(tmp, C_CLIENT)
    return C_CLIENT


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
    print(build_c_client())
