"""Compile the HIP library for gfx950 into paper_2604_18117_amd/liblq.so (in-tree)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
SOURCES = ["lq_api.cpp", "lq_pack_int.hip", "lq_act_int.hip", "lq_fwd_int.hip", "lq_mx.hip", "lq_mx6.hip", "lq_mxi.hip", "lq_calib.hip", "lq_rot.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-ffp-contract=off",
         "-fno-fast-math", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj] + FLAGS
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(extra_flags=()) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(4) as ex:
        objs = list(ex.map(_compile, SOURCES))
    out = os.path.join(HERE, "liblq.so")
    subprocess.run(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", out] + objs, check=True)
    return out


if __name__ == "__main__":
    print(build())
