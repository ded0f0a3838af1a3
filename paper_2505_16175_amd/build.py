"""Builds libqp_hip.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libqp_hip.so")
SOURCES = ["qp_api.hip", "attend_scalar.hip", "attend_mfma.hip", "attend_decode.hip", "score.hip",
           "score_window_mfma.hip", "topk_compact.hip", "gemm_bf16.hip", "gemv_bf16.hip", "layer_kernels.hip", "layer_api.hip", "feed.hip"]


def hipcc_command(out=LIB_PATH, extra=()):
    srcs = [os.path.join(CSRC, s) for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    return ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wall", "-Wno-unused-command-line-argument",
            "-I", os.path.join(ROOT, "include"), "-I", CSRC, *extra, *srcs, "-o", out]


PROBE_PATH = os.path.join(PKG_DIR, "mfma_peak_probe")


def probe_command():
    """The stand-alone matrix-pipe probe (what bf16 MFMA rate this GPU sustains; see bench.py --mfma-probe)."""
    return ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
            "-packed-fp32-ops", "-Wno-unused-command-line-argument", os.path.join(CSRC, "mfma_peak_probe.hip"),
            "-o", PROBE_PATH]


def build(verbose=True):
    for cmd in (hipcc_command(), probe_command()):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    return LIB_PATH


if __name__ == "__main__":
    build()
    print("built", LIB_PATH)
    sys.exit(0)
