"""Builds libe2f.so (HIP, gfx950 only) in-tree next to its sources.

    python -m paper_2601_16622_amd.build          # rebuild everything

Every translation unit is compiled with hipcc for --offload-arch=gfx950 with the packed-fp32 feature switched
off, in parallel, then linked into csrc/libe2f.so.
"""
import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(CSRC, "libe2f.so")
SOURCES = ["e2f_api.hip", "e2f_cells.hip", "e2f_proj.hip", "e2f_fused.hip", "e2f_fused_mfma.hip", "e2f_materialized.hip", "e2f_tp.hip", "e2f_fact.hip", "e2f_tile.hip", "e2f_tile_f32.hip", "e2f_bwd.hip", "e2f_bwd_tile.hip", "e2f_nonlinear.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src):
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = ["hipcc"] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    return src, obj, r.returncode, r.stdout + r.stderr


def build(verbose=True):
    objs = []
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        for src, obj, rc, log in ex.map(_compile, SOURCES):
            log = "\n".join(l for l in log.splitlines() if "packed-fp32-ops" not in l)
            if verbose and log.strip():
                print(f"[{src}]\n{log}")
            if rc != 0:
                raise RuntimeError(f"hipcc failed on {src}")
            objs.append(obj)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
    sys.exit(0)
