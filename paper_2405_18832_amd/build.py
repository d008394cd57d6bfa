"""Build the HIP library in-tree for gfx950: one object per source, one shared library."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libmoe_ffn_gfx950.so")
SOURCES = ["api.hip", "route.hip", "permute.hip", "ffn.hip", "ffn_tile.hip", "combine.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        print(err)
    return obj


def build(verbose: bool = True, defines=(), lib: str = LIB, obj_dir: str = OBJ) -> str:
    """`defines` are extra -D options (tuning constants); `lib`/`obj_dir` name another output."""
    global OBJ
    os.makedirs(obj_dir, exist_ok=True)
    saved, OBJ = OBJ, obj_dir
    extra = [f"-D{d}" for d in defines]
    FLAGS.extend(extra)
    try:
        with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
            objs = list(pool.map(_compile, SOURCES))
    finally:
        OBJ = saved
        del FLAGS[len(FLAGS) - len(extra):]
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    import sys
    defs = [a[2:] for a in sys.argv[1:] if a.startswith("-D")]
    outs = [a for a in sys.argv[1:] if not a.startswith("-D")]
    if outs:
        build(defines=defs, lib=os.path.abspath(outs[0]), obj_dir=os.path.abspath(outs[0]) + ".obj")
    else:
        build(defines=defs)
