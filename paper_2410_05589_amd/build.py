"""Builds libps_draft.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
LIB_PATH = os.path.join(PKG_DIR, "libps_draft.so")
CSRC = os.path.join(PKG_DIR, "csrc")
BUILD_DIR = os.path.join(PKG_DIR, "_build")
HEADERS = [os.path.join(CSRC, "ps_internal.h"), os.path.join(CSRC, "ps_device.h"),
           os.path.join(ROOT, "include", "ps_draft.h"), os.path.join(ROOT, "include", "ps_verify.h"),
           os.path.join(ROOT, "include", "ps_draft_debug.h"), os.path.join(ROOT, "include", "ps_train.h")]
SOURCES = [os.path.join(CSRC, "ps_host.hip"), os.path.join(CSRC, "ps_inst.hip"), os.path.join(CSRC, "ps_verify.hip"),
           os.path.join(CSRC, "ps_measure.hip"), os.path.join(CSRC, "ps_train.hip")]
# the device code is instantiated once per (storage type, head_dim)
INSTANCES = [("f32_d64", 0, 64), ("f32_d128", 0, 128), ("bf16_d64", 1, 64), ("bf16_d128", 1, 128)]


def hipcc_path():
    for p in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc"):
        if p and os.path.exists(p):
            return p
    return "hipcc"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build_library(verbose=True, jobs=4):
    """Compiles every HIP source for gfx950 and links the shared library; always rebuilds."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    common = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc", "-fvisibility=hidden",
              # packed-FP32 instruction selection is switched off for device code
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              # The kernels read their ~1.7 KB parameter struct in hundreds of places.  LLVM replaces the
              # kernel's private copy of the struct by the kernel-argument segment itself only if the copy
              # has at most this many users (default 300); beyond that every parameter read becomes a
              # scratch-memory load and the persistent kernel runs ~40 % slower.
              "-mllvm", "-instcombine-max-copied-from-constant-users=10000",
              "-I", os.path.join(ROOT, "include"), "-I", CSRC] + os.environ.get("PS_BUILD_DEFS", "").split()
    units = [(os.path.join(BUILD_DIR, "ps_host.o"), [os.path.join(CSRC, "ps_host.hip")]),
             (os.path.join(BUILD_DIR, "ps_verify.o"), [os.path.join(CSRC, "ps_verify.hip")]),
             (os.path.join(BUILD_DIR, "ps_measure.o"), [os.path.join(CSRC, "ps_measure.hip")]),
             (os.path.join(BUILD_DIR, "ps_train.o"), [os.path.join(CSRC, "ps_train.hip")])]
    for name, bf, d in INSTANCES:
        units.append((os.path.join(BUILD_DIR, "ps_inst_%s.o" % name),
                      ["-DPS_INST_NAME=%s" % name, "-DPS_INST_BF16=%d" % bf, "-DPS_INST_D=%d" % d,
                       os.path.join(CSRC, "ps_inst.hip")]))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(lambda u: _run(common + ["-c", "-o", u[0]] + u[1], verbose), units))
    out = os.environ.get("PS_BUILD_OUT") or LIB_PATH   # tuning aid: build a variant beside the library
    _run([hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", out]
         + [u[0] for u in units], verbose)
    return out


def library_is_current():
    if not os.path.exists(LIB_PATH):
        return False
    t = os.path.getmtime(LIB_PATH)
    return all(os.path.getmtime(p) <= t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    build_library()
    sys.exit(0)
