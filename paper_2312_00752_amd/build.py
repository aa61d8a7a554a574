"""Build the C-ABI library ``libss_scan.so`` from ``csrc/`` with hipcc for gfx950.

The library is built in-tree (next to this file) so that it travels with the source
tree; nothing is compiled at import time.  ``build_microbench`` builds the stand-alone
ceilings program of ``microbench/`` the same way.
"""
import glob
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libss_scan.so")
BUILD_DIR = os.path.join(PKG, "_build")
MICROBENCH_SRC = os.path.join(PKG, "microbench", "ss_ceilings.hip")
MICROBENCH = os.path.join(PKG, "microbench", "ss_ceilings")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-munsafe-fp-atomics",                     # hardware float atomics, no CAS loops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-FP32 VALU ops
    "-Wno-unused-command-line-argument",
]
PACKED_FP32_OPS = ("v_pk_fma_f32", "v_pk_mul_f32", "v_pk_add_f32")


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _hipcc():
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def _run(cmd, cwd, verbose):
    res = subprocess.run(cmd, cwd=cwd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd))


def _check_no_packed_fp32(directory):
    """The device code must not contain packed-FP32 arithmetic."""
    for asm in glob.glob(os.path.join(directory, "*gfx950*.s")):
        with open(asm) as f:
            text = f.read()
        for op in PACKED_FP32_OPS:
            if op in text:
                raise RuntimeError("%s found in %s" % (op, asm))


def build_library(verbose=False, jobs=None):
    """Compile every .hip source (in parallel) and link libss_scan.so; returns its path."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs = []

    def compile_one(src):
        obj = os.path.join(BUILD_DIR, os.path.basename(src)[:-4] + ".o")
        _run([_hipcc()] + HIPCC_FLAGS + inc + ["-save-temps=obj", "-c", "-o", obj, src], BUILD_DIR, verbose)
        return obj

    with ThreadPoolExecutor(max_workers=jobs or min(8, os.cpu_count() or 1)) as pool:
        objs = list(pool.map(compile_one, sources()))
    _check_no_packed_fp32(BUILD_DIR)
    out = os.path.join(BUILD_DIR, "libss_scan.so")
    _run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + objs, BUILD_DIR, verbose)
    shutil.copy2(out, LIB)
    return LIB


def build_microbench(verbose=False):
    """Compile the stand-alone ceilings program (microbench/ss_ceilings); returns its path."""
    bdir = os.path.join(BUILD_DIR, "microbench")
    os.makedirs(bdir, exist_ok=True)
    out = os.path.join(bdir, "ss_ceilings")
    flags = [f for f in HIPCC_FLAGS if f != "-fPIC"]
    _run([_hipcc()] + flags + ["-save-temps=obj", "-o", out, MICROBENCH_SRC], bdir, verbose)
    _check_no_packed_fp32(bdir)
    shutil.copy2(out, MICROBENCH)
    return MICROBENCH


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_microbench(verbose=True))
