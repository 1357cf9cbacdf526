"""Build libfier.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libfier.so")
SOURCES = ["fier_api.hip", "fier_quantize.hip", "fier_score.hip", "fier_select.hip", "fier_topk.hip",
           "fier_attn.hip", "fier_step.hip", "fier_page.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-mfma-vgpr-form=1",  # matrix-core results stay in ordinary vector registers
         "-I", INCLUDE, "-I", CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s\n%s" % (" ".join(cmd), r.stdout, err))
    if err.strip():
        sys.stderr.write(err + "\n")


def build(verbose: bool = False, prof: bool = False) -> str:
    """Compile every kernel file for gfx950 and link libfier.so next to this file.  Always recompiles.

    prof=True builds the tuning variant libfier_prof.so instead: the same sources with -DFIER_PROF_ENABLE (per-phase
    and per-workgroup time stamps inside the kernels) plus fier_prof.hip, which holds the stamps and exports
    fier_prof_read / fier_prof_read_wg / fier_prof_reset.  Nothing in the product loads it."""
    objdir = os.path.join(HERE, "_build_prof" if prof else "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = _hipcc()
    flags = FLAGS + (["-DFIER_PROF_ENABLE", "-fgpu-rdc"] if prof else [])
    lib = os.path.join(HERE, "libfier_prof.so") if prof else LIB
    jobs = []
    for src in SOURCES + (["fier_prof.hip"] if prof else []):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        jobs.append(([hipcc] + flags + ["-c", os.path.join(CSRC, src), "-o", obj], obj))
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        list(ex.map(lambda j: _run(j[0]), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + (["-fgpu-rdc"] if prof else []) + ["-o", lib] +
         [j[1] for j in jobs])
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    build(verbose=True, prof="--prof" in sys.argv[1:])
