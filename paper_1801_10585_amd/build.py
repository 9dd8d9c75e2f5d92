"""Compile the HIP sources in csrc/ for gfx950 into libscnn.so (in-tree).

hipcc cross-compiles without a GPU.  Objects go to _build/ (ignored by git); the
shared library sits next to this file so that it travels with the tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libscnn.so")
SOURCES = ["scnn_index.hip", "scnn_conv.hip", "scnn_conv_quad.hip", "scnn_topk.hip", "scnn_rows.hip", "scnn_bwd.hip", "scnn_train.hip", "scnn_api.hip"]
# packed fp32 VALU ops are switched off on purpose (they have misbehaved on the target machines)
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-command-line-argument",
         # matrix-core results straight into VGPRs: the fp64 accumulation reads every result once, and a copy out
         # of the accumulation registers would cost one more vector instruction per value
         "-mllvm", "-amdgpu-mfma-vgpr-form"]


def _deps_mtime() -> float:
    paths = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", "scnn.h")]
    return max(os.path.getmtime(p) for p in paths)


def is_stale() -> bool:
    return not os.path.exists(LIB) or os.path.getmtime(LIB) < _deps_mtime()


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(BUILD, src.replace(".hip", ".o"))
    src_path = os.path.join(CSRC, src)
    hdr_m = max(os.path.getmtime(os.path.join(CSRC, "scnn_internal.h")),
                os.path.getmtime(os.path.join(HERE, "..", "include", "scnn.h")))
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= max(os.path.getmtime(src_path), hdr_m):
        return obj
    cmd = ["hipcc", *FLAGS, "-c", src_path, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("hipcc failed on " + src)
    return obj


def build(force: bool = True, jobs: int = 7) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("link failed")
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))
