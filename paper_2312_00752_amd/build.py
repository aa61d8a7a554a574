"""Build the C-ABI library ``libss_scan.so`` from ``csrc/`` with hipcc for gfx950.

The library is built in-tree (next to this file) so that it travels with the source
tree; nothing is compiled at import time.
"""
import glob
import os
import shutil
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libss_scan.so")
BUILD_DIR = os.path.join(PKG, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-munsafe-fp-atomics",                     # hardware float atomics, no CAS loops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-FP32 VALU ops
    "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_library(verbose=False):
    """Compile every .hip source into libss_scan.so; returns its path."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    os.makedirs(BUILD_DIR, exist_ok=True)
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC,
                                  "-save-temps=obj", "-o", os.path.join(BUILD_DIR, "libss_scan.so")] + sources()
    res = subprocess.run(cmd, cwd=BUILD_DIR, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed")
    # the device code must not contain packed-FP32 arithmetic
    for asm in glob.glob(os.path.join(BUILD_DIR, "*gfx950*.s")):
        with open(asm) as f:
            text = f.read()
        for op in ("v_pk_fma_f32", "v_pk_mul_f32", "v_pk_add_f32"):
            if op in text:
                raise RuntimeError("%s found in %s" % (op, asm))
    shutil.copy2(os.path.join(BUILD_DIR, "libss_scan.so"), LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
