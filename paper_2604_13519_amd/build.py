"""Builds libtoolspec_hip.so (gfx950) in-tree with hipcc.

    python -m paper_2604_13519_amd.build

The library has no Python or PyTorch dependency: it links against the HIP runtime
only and is loaded through ctypes by binding.py.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libtoolspec_hip.so")
SOURCES = ["ts_host.hip", "ts_kernels_misc.hip", "ts_gemm_bf16.hip", "ts_gemm_rows_bf16.hip", "ts_attn_bf16.hip", "ts_draft.cpp", "ts_generate.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # keep hipcc from forming packed-fp32 instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build_library(verbose=True):
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = _hipcc()
    objs = [os.path.join(OBJ_DIR, os.path.splitext(s)[0] + ".o") for s in SOURCES]

    def compile_one(pair):
        src, obj = pair
        inc = ["-I", os.path.join(os.path.dirname(HERE), "include")]
        if src.endswith(".cpp"):                       # host-only C++ (drafting): no device pass
            cmd = [hipcc, "-x", "c++", "-O2", "-std=c++17", "-fPIC"] + inc
        else:
            cmd = [hipcc] + FLAGS + inc
        out = _run(cmd + ["-c", os.path.join(CSRC, src), "-o", obj])
        if verbose and out.strip():
            print(out)
        return obj

    with ThreadPoolExecutor(4) as ex:
        list(ex.map(compile_one, zip(SOURCES, objs)))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objs)
    if verbose:
        print("built", LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    build_library()
    sys.exit(0)
