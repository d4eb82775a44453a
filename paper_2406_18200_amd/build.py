"""Builds libseed_verify.so (gfx950) in-tree with hipcc.  Usage: python -m paper_2406_18200_amd.build

Every source is compiled to an object of its own (in parallel, under _build/, which is not tracked) and the
objects are linked into the one shared library next to this file."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libseed_verify.so")
SOURCES = ["seed_api.hip", "accept.hip", "gemm_bf16.hip", "rowops.hip", "attention_bf16.hip", "fp32_path.hip",
           "sched.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose=True, jobs=None, changed_only=False):
    """changed_only: recompile only the sources (or headers) newer than their object; the default compiles all."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    sources = list(SOURCES)
    cflags = [f for f in FLAGS if f != "-shared"]
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in sources]
    cmds = [[hipcc] + cflags + ["-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(sources, objs)]
    if changed_only:
        hdr = max(os.path.getmtime(os.path.join(d, f)) for d in (CSRC, os.path.join(HERE, "..", "include"))
                  for f in os.listdir(d) if f.endswith(".h"))
        cmds = [c for c, s, o in zip(cmds, sources, objs)
                if not os.path.exists(o) or os.path.getmtime(o) < max(hdr, os.path.getmtime(os.path.join(CSRC, s)))]
    jobs = jobs or max(1, min(len(cmds), int(os.environ.get("MAX_JOBS", "8"))))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc"] + objs + ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    build(changed_only="--changed" in sys.argv[1:])
    sys.exit(0)
