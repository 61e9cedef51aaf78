"""Builds libvlcache.so (hand-written HIP kernels + the C-ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libvlcache.so")

SOURCES = ["api.hip", "score_simple.hip", "score_mfma.hip", "window_attn.hip", "window_attn_simple.hip", "allocate.hip", "topk_compact.hip", "decode.hip", "probe.hip"]

# packed fp32 VALU ops are switched off for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", *os.environ.get("VLC_EXTRA_FLAGS", "").split(), "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # one-lane atomics whose result is needed much later: do not let the compiler turn them into a wave-wide
         # reduction that waits for the result at once
         "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(ln for ln in p.stdout.splitlines() if "is not a recognized feature for this target" not in ln)
    if p.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False, incremental: bool = False) -> str:
    """Compiles every source (incremental=True, a developer convenience: only those older than their object
    file or than any header) and links the shared library."""
    os.makedirs(BUILD, exist_ok=True)
    hipcc = _hipcc()
    srcs = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")] + \
              [os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))] + [os.path.abspath(__file__)]
    newest_header = max(os.path.getmtime(h) for h in headers)

    def compile_one(src):
        obj = os.path.join(BUILD, src.replace(".hip", ".o"))
        path = os.path.join(CSRC, src)
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(path), newest_header):
            return obj, ""
        out = _run([hipcc, *FLAGS, "-c", path, "-o", obj])
        return obj, out

    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        results = list(ex.map(compile_one, srcs))
    for obj, out in results:
        if verbose and out.strip():
            print(out)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *[o for o, _ in results]])
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, incremental="-i" in sys.argv))
