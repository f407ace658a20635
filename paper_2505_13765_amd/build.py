"""Builds libwind.so (the C-ABI library) with hipcc for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libwind.so")
SOURCES = ["wind_api.hip"]
DEPS = ["wind_api.hip", "wind_kernels.h", "wind_types.h", "wind_enc_kernels.h", "wind_joint_kernels.h", "wind_decide_kernels.h",
        "wind_pred_kernels.h", "wind_loop_kernel.h", "wind_mfma.h", "wind_mfma_dma.h", "wind_mfma_ws.h", "wind_mfma_wide.h", "wind_util.h", "wind_beam.h",
        "wind_beam_search.h", os.path.join("..", "..", "include", "wind.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, d)) > t for d in DEPS)


def build(force: bool = True) -> str:
    """Compile every HIP source into paper_2505_13765_amd/libwind.so."""
    if force or stale():
        cmd = ["hipcc", *FLAGS, "-o", LIB, *[os.path.join(CSRC, s) for s in SOURCES]]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(True))
