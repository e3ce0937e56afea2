"""Builds libssam.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

Every translation unit under csrc/ is compiled to an object (in parallel) and linked into
paper_1907_06154_amd/libssam.so.  Packed-FP32 instruction selection is disabled on the
device side, as required on the test machines.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libssam.so")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # matrix-core accumulators stay in ordinary vector registers: the lane shifts read them there, and
         # the moves to and from the accumulation registers cost 3-7 % on the 7x7 ... 20x20 filters
         "-mllvm", "-amdgpu-mfma-vgpr-form=1",
         "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes"]


def _up_to_date(obj: str) -> bool:
    """True when obj is newer than every file its dependency list (written by -MD) names."""
    dep = obj + ".d"
    if not (os.path.exists(obj) and os.path.exists(dep)):
        return False
    t = os.path.getmtime(obj)
    words = open(dep).read().replace("\\\n", " ").split()
    files = [w for w in words[1:] if not w.endswith(":")]
    return all(os.path.exists(f) and os.path.getmtime(f) <= t for f in files)


def _compile(src: str, extra, incremental: bool = False) -> str:
    # objects of a build with extra defines live in a folder of their own
    objdir = OBJ if not extra else OBJ + "_" + "".join(c if c.isalnum() else "_" for c in "".join(extra))
    os.makedirs(objdir, exist_ok=True)
    obj = os.path.join(objdir, os.path.basename(src) + ".o")
    if incremental and _up_to_date(obj):
        return obj
    cmd = ["hipcc", *FLAGS, *extra, "-MD", "-MF", obj + ".d", "-c", src, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{res.stdout}\n{res.stderr}")
    noise = "is not a recognized feature for this target"   # host pass does not know the device feature
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False, jobs: int = 8, extra=(), lib: str = LIB, incremental: bool = False) -> str:
    """incremental: recompile only the translation units whose sources or headers changed since
    their object was written (a developer's shortcut; the default compiles everything)."""
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(lambda s: _compile(s, list(extra), incremental), srcs))
    link_extra = [a for a in extra if "sanitize" in a]      # a sanitizer build links its runtime too
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *link_extra, "-o", lib, *objs]
    subprocess.run(cmd, check=True)
    if verbose:
        print(f"built {lib} from {len(srcs)} translation units")
    return lib


if __name__ == "__main__":
    # python -m paper_1907_06154_amd.build [output.so] [-DNAME ...] [--incremental] [--sanitize-host]
    #   -DNAME: extra defines (experiments).  --sanitize-host: AddressSanitizer + UBSan on the HOST code only
    #   (validation, planner, dispatch; device code is compiled as usual), for a CPU run of the host-only
    #   tests with clang's asan runtime preloaded.
    args = sys.argv[1:]
    out = next((a for a in args if a.endswith(".so")), LIB)
    extra = [a for a in args if a.startswith("-D")]
    if "--sanitize-host" in args:
        extra += ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
                  "-fno-omit-frame-pointer", "-g"]
    build(verbose=True, extra=extra, lib=out, incremental="--incremental" in args)
