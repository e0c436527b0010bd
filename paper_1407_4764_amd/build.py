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


# Host-side sanitizer builds (CPU only): the argument validation, workspace layout and switches of
# otf_api.hip are host code; these flags instrument that code and leave the device code alone.
HOST_SANITIZERS = {
    # no runtime library needed, so the result can be loaded into any process: undefined behaviour traps
    "ubsan-trap": ["-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fsanitize-trap=undefined"],
    # needs the sanitizer runtime first in the process: for executables of our own
    "asan-ubsan": ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                   "-Xarch_host", "-fno-sanitize-recover=undefined"],
}


def build_host_checked(kind, driver=None):
    """otf_api.hip rebuilt with HOST_SANITIZERS[kind] and linked with the ordinary objects of the
    other sources: into _build/libotf_<kind>.so, or, with `driver` (a C++ source that calls the C
    ABI), into the executable _build/<driver name>_<kind>.  Returns the path."""
    os.makedirs(BUILD, exist_ok=True)
    others = []
    for src in SOURCES:
        if src == "otf_api.hip":
            continue
        obj = os.path.join(BUILD, src.replace(".hip", ".o"))
        if not os.path.exists(obj) or os.path.getmtime(obj) < os.path.getmtime(os.path.join(CSRC, src)):
            obj = _compile(src)
        others.append(obj)
    api = os.path.join(BUILD, "otf_api.%s.o" % kind)
    cmd = ["hipcc"] + FLAGS + ["-O1", "-g"] + HOST_SANITIZERS[kind] + ["-c", os.path.join(CSRC, "otf_api.hip"), "-o", api]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on otf_api.hip (%s):\n%s" % (kind, r.stdout + r.stderr))
    if driver is None:
        out = os.path.join(BUILD, "libotf_%s.so" % kind)
        cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, api] + others
    else:
        out = os.path.join(BUILD, "%s_%s" % (os.path.splitext(os.path.basename(driver))[0], kind))
        cmd = ["hipcc", "--offload-arch=gfx950", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
               "-fno-sanitize-recover=undefined", "-fno-gpu-sanitize", "-I" + INCLUDE, "-x", "c++", driver,
               "-x", "none", api] + others + ["-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed (%s):\n%s" % (kind, r.stdout + r.stderr))
    return out


if __name__ == "__main__":
    print(build_library())
