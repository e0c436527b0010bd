"""Builds paper_1407_4764_amd/libotf.so from csrc/*.hip with hipcc for gfx950 (cross-compiles
without a GPU).  Usage: python -m paper_1407_4764_amd.build"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libotf.so")

SOURCES = ["otf_api.hip", "otf_select.hip", "otf_dense.hip", "otf_table.hip", "otf_mfma.hip", "otf_sgd.hip", "otf_encode.hip",
           "otf_pq_train.hip", "otf_sparse.hip"]
# packed-fp32 instructions are switched off for every device translation unit
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-I" + INCLUDE, "-I" + CSRC, "-Wall", "-Wno-unused-function"]
# The matrix-core scan orders its next tile with a one-lane atomic whose result it reads two steps
# later.  The compiler's wave-aggregation of atomics would insert a read of the result (and a full
# memory wait) right behind the atomic, so it is switched off for that file.
# The scan that walks long rows through several table images orders its next block the same way.
NO_ATOMIC_AGGREGATION = ["-mllvm", "-amdgpu-atomic-optimizer-strategy=None"]
EXTRA_FLAGS = {"otf_mfma.hip": NO_ATOMIC_AGGREGATION, "otf_table.hip": NO_ATOMIC_AGGREGATION}


def _compile(src):
    obj = os.path.join(BUILD, src.replace(".hip", ".o"))
    cmd = ["hipcc"] + FLAGS + EXTRA_FLAGS.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                     if "is not a recognized feature for this target" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, msgs))
    if msgs.strip():
        sys.stderr.write(msgs + "\n")
    return obj


def build_library(jobs=6):
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build_library())
