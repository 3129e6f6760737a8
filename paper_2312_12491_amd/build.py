"""Builds libsdstream.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libsdstream.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wno-unused-result", "-Wno-unused-value",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]
# SDSTREAM_DEVHOOKS=1 in the environment of the BUILD compiles in the environment-variable switches used for kernel
# sweeps (SDSTREAM_TUNE, SDSTREAM_ATTN_QT, SDSTREAM_NO_MFMA, SDSTREAM_PROFILE_OPS); the normal library reads none.
if os.environ.get("SDSTREAM_DEVHOOKS") == "1":
    FLAGS.append("-DSDSTREAM_DEVHOOKS")


# per-file additions.  attn_mfma: without NaNs to honour, fmaxf needs no canonicalising v_max x, x, x in front of it
# (28 vector instructions per key tile in a kernel that is bound by them; masked scores are -3e38, never NaN)
EXTRA = {"attn_mfma.hip": ["-fno-honor-nans"]}


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src[:-4] + ".o")
    cmd = [HIPCC] + FLAGS + EXTRA.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(only_stale: bool = False, jobs: int = 8) -> str:
    """Compiles every csrc/*.hip and links the shared library.  only_stale skips objects newer than all sources."""
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")] + \
              [os.path.join(ROOT, "include", "sdstream.h")]
    newest_h = max(os.path.getmtime(h) for h in headers)
    todo = []
    for s in srcs:
        obj = os.path.join(OBJ, s[:-4] + ".o")
        if only_stale and os.path.exists(obj) and os.path.getmtime(obj) > max(newest_h, os.path.getmtime(os.path.join(CSRC, s))):
            continue
        todo.append(s)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(_compile, todo))
    objs = [os.path.join(OBJ, s[:-4] + ".o") for s in srcs]
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs,
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(only_stale="--stale" in sys.argv))
