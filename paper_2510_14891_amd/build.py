"""Builds the C-ABI HIP library in-tree for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "mttkrp.hip")
SRC_ABLATION = os.path.join(HERE, "csrc", "ablation.hip")
SRC_CPALS = os.path.join(HERE, "csrc", "cpals.hip")
SRC_CALIBRATE = os.path.join(HERE, "csrc", "calibrate.hip")
HEADER = os.path.join(os.path.dirname(HERE), "include", "mttkrp.h")
HEADER_ABLATION = os.path.join(os.path.dirname(HERE), "include", "mttkrp_ablation.h")
LIB = os.path.join(HERE, "libmttkrp_hip.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # hipcc must not form packed-fp32 VALU ops on these machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile csrc/mttkrp.hip into libmttkrp_hip.so next to this file."""
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= max(os.path.getmtime(SRC), os.path.getmtime(HEADER),
                                             os.path.getmtime(SRC_ABLATION), os.path.getmtime(HEADER_ABLATION),
                                             os.path.getmtime(SRC_CPALS), os.path.getmtime(SRC_CALIBRATE),
                                             os.path.getmtime(os.path.join(HERE, "csrc", "gen_pipe.py")),
                                             os.path.getmtime(os.path.join(HERE, "csrc", "gen_rows_pipe.py")))):
        return LIB
    # write the inline-assembly includes (deterministic build products of the two generators)
    for gen in ("gen_pipe.py", "gen_rows_pipe.py"):
        subprocess.run([sys.executable, os.path.join(HERE, "csrc", gen)], check=True, stdout=subprocess.DEVNULL)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB, SRC, SRC_ABLATION, SRC_CPALS, SRC_CALIBRATE]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(force=True, verbose=True)
    print(LIB)
