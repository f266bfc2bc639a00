"""Build the HIP library for gfx950 with hipcc (cross-compiles without a GPU)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkfac_mi355x.so")
SOURCES = ["kfac_hip.hip", "bubble_fill.cpp"]
HEADERS = ["tn_gemm.h", "diag_block.h", "bf16_syrk256.h", "split3_syrk256.h", "split2_syrk256.h", "mfma_probe.h", os.path.join("..", "..", "include", "kfac.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    # keep the compiler from forming packed fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the direct-to-LDS loads set m0 inside their asm statement and name it as clobbered; the compiler warns
    # about that once per expansion (thousands of lines), which hides every other message
    "-Wno-inline-asm",
]


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    files = [os.path.join(CSRC, s) for s in SOURCES + HEADERS]
    return any(os.path.getmtime(f) > t for f in files)


def build(force=True, verbose=False):
    """Compile ``libkfac_mi355x.so`` in-tree; returns its path."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
