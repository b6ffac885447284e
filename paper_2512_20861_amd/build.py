"""Build step: compile the HIP sources in csrc/ into libblr.so for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libblr.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))


def _run(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    return err


def build_library(verbose: bool = False) -> str:
    """Compile every kernel translation unit (in parallel) and link the C-ABI shared library in-tree."""
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    srcs = sources()
    with tempfile.TemporaryDirectory(prefix="blr_build_") as tmp:
        objs = [os.path.join(tmp, os.path.basename(src) + ".o") for src in srcs]
        compile_flags = [f for f in FLAGS if f != "-shared"]
        with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as pool:
            errs = list(pool.map(lambda so: _run([HIPCC] + compile_flags + ["-c", so[0], "-o", so[1]]), zip(srcs, objs)))
        errs.append(_run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB]))
    if verbose and any(e.strip() for e in errs):
        print("\n".join(e for e in errs if e.strip()))
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
