"""Builds libps_draft.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
LIB_PATH = os.path.join(PKG_DIR, "libps_draft.so")
SOURCES = [os.path.join(PKG_DIR, "csrc", n) for n in ("ps_host.hip", "ps_kernels.hip")]
HEADERS = [os.path.join(PKG_DIR, "csrc", "ps_internal.h"), os.path.join(ROOT, "include", "ps_draft.h")]


def hipcc_path():
    for p in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc"):
        if p and os.path.exists(p):
            return p
    return "hipcc"


def build_library(verbose=True):
    """Compiles every HIP source for gfx950; always rebuilds."""
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-fno-gpu-rdc",
           # packed-FP32 instruction selection is switched off for device code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG_DIR, "csrc"),
           "-o", LIB_PATH] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB_PATH


def library_is_current():
    if not os.path.exists(LIB_PATH):
        return False
    t = os.path.getmtime(LIB_PATH)
    return all(os.path.getmtime(p) <= t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    build_library()
    sys.exit(0)
