"""Compile the HIP sources of the rollout library for gfx950 into one shared library, in-tree.

Usage: python -m paper_2510_17891_amd.build [--force]
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "librl_rollout.so")
SOURCES = ["small_kernels.hip", "gemm_bf16.hip", "attn_bf16.hip", "generic_f32.hip", "sampler.hip", "objective.hip", "model.hip"]
HEADERS = ["device_utils.h", "kernels.h", "seq_table.h", "sampler_device.h", "attn_plan.h", "rope_device.h", "weight_order.h", os.path.join("..", "..", "include", "rl.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _newest_header():
    return max(os.path.getmtime(os.path.join(CSRC, h)) for h in HEADERS)


def _compile(src, force):
    s = os.path.join(CSRC, src)
    o = os.path.join(OBJ, src.replace(".hip", ".o"))
    if (not force and os.path.exists(o)
            and os.path.getmtime(o) >= max(os.path.getmtime(s), _newest_header())):
        return o, False
    subprocess.run(["hipcc", *FLAGS, "-c", s, "-o", o], check=True)
    return o, True


def build(force: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=6) as ex:
        res = list(ex.map(lambda s: _compile(s, force), SOURCES))
    objs = [o for o, _ in res]
    if force or any(c for _, c in res) or not os.path.exists(LIB):
        subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
