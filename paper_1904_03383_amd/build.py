"""Build libtgemm.so (HIP kernels + C-ABI) for gfx950 with hipcc, in-tree.

    python -m paper_1904_03383_amd.build            # rebuild what changed
    python -m paper_1904_03383_amd.build --force    # rebuild everything
    python -m paper_1904_03383_amd.build --poison   # also the debug flavour libtgemm_poison.so (TG_POISON_LDS:
                                                    # LDS stages are overwritten with NaN once they are given up)
"""
from __future__ import annotations

import concurrent.futures
import os
import pathlib
import subprocess
import sys

PKG = pathlib.Path(__file__).resolve().parent
CSRC = PKG / "csrc"
OBJ = PKG / "_build"
LIB = PKG / "libtgemm.so"
OBJ_POISON = PKG / "_build_poison"
LIB_POISON = PKG / "libtgemm_poison.so"

ARCH = "gfx950"
# -packed-fp32-ops is switched off: the compiler must not form packed fp32 instructions.
COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
HIP_FLAGS = [f"--offload-arch={ARCH}"] + COMMON


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def sources():
    return sorted(CSRC.glob("*.hip")) + sorted(CSRC.glob("*.cpp"))


def _headers_mtime() -> float:
    hdrs = list(CSRC.glob("*.h")) + list(CSRC.glob("*.hpp")) + [PKG.parent / "include" / "tgemm.h"]
    return max(h.stat().st_mtime for h in hdrs)


def _compile(src: pathlib.Path, force: bool, hdr_mtime: float, objdir: pathlib.Path = OBJ, defines=()) -> pathlib.Path:
    obj = objdir / (src.name + ".o")
    if not force and obj.exists() and obj.stat().st_mtime > max(src.stat().st_mtime, hdr_mtime):
        return obj
    cmd = [_hipcc()] + HIP_FLAGS + [f"-D{d}" for d in defines] + ["-c", str(src), "-o", str(obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"{' '.join(cmd)}\n{r.stdout}\n{r.stderr}")
    return obj


def build(force: bool = False, jobs: int | None = None, poison: bool = False) -> pathlib.Path:
    """Compile and link the library; with poison=True the debug flavour (its own object folder and file name)."""
    objdir = OBJ_POISON if poison else OBJ
    LIB = LIB_POISON if poison else globals()["LIB"]
    defines = ("TG_POISON_LDS",) if poison else ()
    objdir.mkdir(exist_ok=True)
    srcs = sources()
    hdr_mtime = _headers_mtime()
    jobs = jobs or min(8, len(srcs), os.cpu_count() or 1)
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, hdr_mtime, objdir, defines), srcs))
    if force or not LIB.exists() or LIB.stat().st_mtime < max(o.stat().st_mtime for o in objs):
        # The library needs libamdhip64.so.7 by soname: inside a PyTorch process it binds to the
        # runtime torch has already loaded (the binding imports torch first; two HIP runtimes in
        # one process do not both see the GPU), stand-alone it finds ROCm's through the run path.
        cmd = [_hipcc(), f"--offload-arch={ARCH}", "-shared", "-fPIC", "-o", str(LIB)] + [str(o) for o in objs]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"{' '.join(cmd)}\n{r.stdout}\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
    if "--poison" in sys.argv:
        print(build(force="--force" in sys.argv, poison=True))
