"""Compiles the HIP sources of this package into libsageattn.so (gfx950 only), in-tree."""
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
SOURCES = ["sage_api.hip", "sage_prologue.hip", "sage_attn_kernel.hip"]
LIB = os.path.join(PKG, "libsageattn.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed FP32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build_library(verbose=True, extra_flags=(), out=LIB):
    srcs = [os.path.join(PKG, "csrc", s) for s in SOURCES]
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(PKG, "csrc"), "-o", out, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(ln for ln in res.stdout.splitlines()
                    if "packed-fp32-ops" not in ln and "is not a recognized feature" not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return out


ABI_SMOKE_SRC = os.path.join(ROOT, "tests", "abi_c", "abi_smoke.c")
ABI_SMOKE_BIN = os.path.join(ROOT, "tests", "abi_c", "abi_smoke")


def build_abi_smoke(verbose=True):
    """Compiles tests/abi_c/abi_smoke.c, a plain-C caller of the library (host compiler, no HIP device code)."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-O2", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
           "-I", os.path.join(ROOT, "include"), "-o", ABI_SMOKE_BIN, ABI_SMOKE_SRC,
           "-L", PKG, "-l:libsageattn.so", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../../paper_2411_10958_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("gcc failed:\n" + res.stdout)
    return ABI_SMOKE_BIN


PROBE_SRC = os.path.join(PKG, "csrc", "probe_valu_issue.hip")
PROBE_BIN = os.path.join(PKG, "probe_valu_issue")


def build_probe(verbose=True):
    """Compiles csrc/probe_valu_issue.hip, the stand-alone hardware probe the vector-ALU ceiling quoted by bench.py
    comes from (profiles/valu_issue_probe.txt holds its output)."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O2", "-std=c++17", "-Wno-unused-command-line-argument", "-o", PROBE_BIN, PROBE_SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    return PROBE_BIN


if __name__ == "__main__":
    build_library(extra_flags=sys.argv[1:])
    build_abi_smoke()
    build_probe()
