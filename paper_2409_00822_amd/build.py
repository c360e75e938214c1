"""Build librtopk.so (HIP, gfx950) in-tree.  Run as `python -m paper_2409_00822_amd.build`."""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "librtopk.so")

SOURCES = ["rtopk_api.hip", "rtopk_inst_g4_exact.hip", "rtopk_inst_g4_early.hip", "rtopk_inst_g4_eps.hip",
           "rtopk_inst_small.hip", "rtopk_inst_h16_exact.hip", "rtopk_inst_h16_early.hip", "rtopk_inst_dense.hip", "rtopk_inst_block.hip", "rtopk_inst_block_var.hip",
           "rtopk_inst_block_dense.hip", "rtopk_inst_block_h16.hip", "rtopk_inst_backward.hip", "rtopk_inst_stream.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",          # the fp32 midpoint must round exactly like a scalar CPU evaluation
    "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    subprocess.check_call(cmd)
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    # regenerate the inline-assembly search loops (a no-op when the committed file is current)
    subprocess.check_call([sys.executable, os.path.join(CSRC, "gen_search_loops.py")], stdout=subprocess.DEVNULL)
    with concurrent.futures.ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH])
    if verbose:
        print("built", LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
