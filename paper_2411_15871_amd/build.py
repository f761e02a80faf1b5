"""Builds libdhelix.so for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_2411_15871_amd.build [--force]
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdhelix.so")
SOURCES = ["api.cpp", "plan.cpp", "rowops.hip", "standin.hip", "gemm_f32.hip", "gemm_bf16.hip", "attn_f32.hip",
           "attn_bf16.hip", "moe.hip", "layer.hip", "stack.cpp"]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
         "-Wno-unknown-warning-option", "-Wno-inline-asm"]
# Per-source additions.  attn_bf16.hip: matrix instructions issued through the intrinsic write ordinary registers
# (its long-lived accumulators are placed in AGPRs by hand); no NaN ever enters a max/min there.
EXTRA_FLAGS = {"attn_bf16.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form", "-fno-honor-nans"]}


def _deps_mtime():
    hdrs = [os.path.join(CSRC, "common.h"), os.path.join(HERE, "..", "include", "dhelix.h")]
    return max(os.path.getmtime(h) for h in hdrs)


def _compile(src, force):
    obj = os.path.join(OBJ, src + ".o")
    path = os.path.join(CSRC, src)
    if not force and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(path), _deps_mtime()):
        return obj, ""
    r = subprocess.run(["hipcc"] + FLAGS + EXTRA_FLAGS.get(src, []) + ["-c", path, "-o", obj], capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, msgs))
    return obj, msgs


def build(force=True, verbose=False):
    """Compiles every source and links libdhelix.so.  force=False reuses up-to-date objects."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        results = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if verbose:
        for _, m in results:
            if m.strip():
                print(m)
    objs = [o for o, _ in results]
    r = subprocess.run(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs,
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
