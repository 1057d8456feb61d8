"""Compile csrc/*.hip into paper_2407_12820_amd/libpqcache.so for gfx950.

hipcc cross-compiles without a GPU.  Packed-fp32 instructions are switched off for
all device code (-Xclang -target-feature -Xclang -packed-fp32-ops); the host pass
warns that it does not know that feature, which is harmless.
"""
import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpqcache.so")
OBJ = os.path.join(HERE, "_build")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-command-line-argument",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # keep returning atomics as written: the wave-level rewrite reads the result back at once,
         # which puts the atomic's round trip on the critical path of select_kernel
         "-mllvm", "-amdgpu-atomic-optimizer-strategy=None"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _compile(src: str, defines=(), obj_dir: str = OBJ) -> str:
    obj = os.path.join(obj_dir, os.path.basename(src) + ".o")
    r = subprocess.run(["hipcc", *FLAGS, *[f"-D{d}" for d in defines], "-c", src, "-o", obj], capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        print(err)
    return obj


def build(jobs: int = 8, defines=(), out: str = LIB) -> str:
    """Compile and link the library.  `defines` are build switches of the sources (e.g. PQC_VECTOR_ATTENTION: the
    vector-ALU attention for bf16 caches, kept for comparison measurements); a build with switches goes to `out`,
    which must then differ from the default library path."""
    if defines and os.path.abspath(out) == os.path.abspath(LIB):
        raise ValueError("a build with switches needs its own output path")
    obj_dir = OBJ if not defines else OBJ + "_" + "_".join(sorted(defines))
    os.makedirs(obj_dir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(lambda s: _compile(s, defines, obj_dir), sources()))
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", out],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return out


if __name__ == "__main__":
    import argparse

    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--define", action="append", default=[], help="build switch, e.g. PQC_VECTOR_ATTENTION")
    ap.add_argument("--out", default=LIB, help="output library (required with --define)")
    a = ap.parse_args()
    print(build(defines=tuple(a.define), out=a.out))
