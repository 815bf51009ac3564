"""Build step: compile the HIP sources of the hot path into one shared library for gfx950.

    python -m paper_2601_17917_amd.build [--incremental]

hipcc cross-compiles without a GPU.  Every source is compiled to an object of its own (in parallel,
under _build/, git-ignored) and the objects are linked into libsdllm.so next to this file (git-ignored;
it travels with the tree).  --incremental skips sources whose object is newer than the source and every
header; the default compiles everything."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsdllm.so")
SOURCES = ["api.hip", "kv_append.hip", "unmask.hip", "attention_f32.hip", "attention_bf16.hip", "rope.hip",
           "lm_head.hip", "probe.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wno-inline-asm",
    # packed fp32 VALU forms are kept off for every HIP source of this build
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless, filtered
    err = "\n".join(ln for ln in res.stderr.splitlines() if "packed-fp32-ops" not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stdout + "\n" + res.stderr)
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build(verbose: bool = True, incremental: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    headers = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)
    jobs = []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s + ".o")
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            continue
        jobs.append([hipcc] + FLAGS + ["-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as ex:
        list(ex.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + [os.path.join(OBJ, s + ".o") for s in SOURCES]
         + ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    print(build(incremental="--incremental" in sys.argv[1:]))
