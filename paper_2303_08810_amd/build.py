"""Builds libbra.so (HIP, gfx950 only) in-tree with hipcc: one compile per source file, in
parallel, then one link."""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbra.so")
OBJ_DIR = os.path.join(HERE, "_build")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # packed float32 VALU instructions stay off (hipcc would otherwise form them)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def compile_objects(tag="product", defines=(), extra_flags=(), opt="-O3", verbose=False, jobs=None):
    """One object file per source, compiled in parallel; returns their paths."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    obj_dir = os.path.join(OBJ_DIR, tag)
    os.makedirs(obj_dir, exist_ok=True)
    flags = [f if f != "-O3" else opt for f in HIPCC_FLAGS] + ["-D" + d for d in defines] + list(extra_flags)

    def compile_one(src):
        obj = os.path.join(obj_dir, os.path.basename(src)[:-4] + ".o")
        cmd = [hipcc] + flags + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True, cwd=CSRC, stdout=subprocess.PIPE, stderr=subprocess.STDOUT if not verbose else None)
        return obj

    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        return list(pool.map(compile_one, sources()))


def build(verbose: bool = False, out: str = LIB, defines=(), jobs: int | None = None) -> str:
    """Always recompiles.  `defines`: extra -D names (BRA_EXPERIMENT makes the A/B switches of
    the kernels readable from the environment; the shipped library is built without it)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = compile_objects(tag="_".join(defines) or "product", defines=defines, verbose=verbose, jobs=jobs)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, cwd=CSRC)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
