"""Compile the HIP sources into libpsd.so for gfx950 (in-tree, next to this file).

`python -m paper_2510_26527_amd.build`; hipcc cross-compiles without a GPU.

The library is linked against the HIP runtime that PyTorch ships and loads
(soname libamdhip64.so), not against a second copy: device pointers and streams
handed over from torch tensors must belong to the same runtime instance.
"""
import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
OBJ = os.path.join(_HERE, "_build")
LIB = os.path.join(_HERE, "libpsd.so")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-value", "-Wno-unknown-attributes"]
_NOISE = "is not a recognized feature for this target"


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if _NOISE not in l)
    if r.returncode != 0:
        raise RuntimeError(" ".join(cmd) + "\n" + err)
    return err


def _torch_lib_dir():
    import torch
    return os.path.join(os.path.dirname(torch.__file__), "lib")


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    objs = []
    jobs = []
    for src in sources():
        obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        jobs.append(["hipcc"] + FLAGS + ["-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        for cmd, err in zip(jobs, ex.map(_run, jobs)):
            if verbose:
                print(" ".join(cmd))
                if err.strip():
                    print(err)
    tl = _torch_lib_dir()
    link = ["g++", "-shared", "-o", LIB] + objs + ["-L" + tl, "-lamdhip64", "-Wl,-rpath," + tl,
                                                   "-Wl,-rpath,/opt/rocm/lib"]
    _run(link)
    if verbose:
        print(" ".join(link))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
