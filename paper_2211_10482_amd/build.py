"""Build libstructtensor_hip.so (HIP kernels + C ABI) for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libstructtensor_hip.so")
SOURCES = ["st_api.hip", "st_expand.hip", "st_batax.hip", "st_ttm.hip", "st_moment3.hip", "st_mttkrp.hip",
           "st_moment2.hip", "st_moment4.hip", "st_moment_mfma.hip", "st_covar_small.hip", "st_table.hip", "st_desc.hip",
           "st_probe.hip"]
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
]
API_VISIBILITY = ["-fvisibility=default"]  # st_api.hip and st_desc.hip export the extern "C" entry points


def _compile(src: str, extra=()) -> str:
    obj = os.path.join(BUILD, src.replace(".hip", ".o"))
    flags = list(FLAGS)
    if src in ("st_api.hip", "st_desc.hip"):
        flags = [f for f in flags if f != "-fvisibility=hidden"] + API_VISIBILITY
    cmd = ["hipcc", *flags, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, r.stderr))
    warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if "warning" in warn:
        print(warn)
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs, "-lhiprtc"]
    subprocess.run(cmd, check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
