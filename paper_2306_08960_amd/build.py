"""Build libapb.so (the C-ABI HIP library) in-tree for gfx950 with hipcc.

Every source is compiled to an object of its own (in parallel), then the objects are linked; the
objects live under _build/ at the repository root.  `build(force=True)` recompiles everything,
`build(force=False)` only the sources that are newer than their object (a header change recompiles
everything)."""
from __future__ import annotations

import concurrent.futures
import glob
import os
import subprocess
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libapb.so")
SOURCES = ["apb_api.hip", "apb_compress.hip", "apb_quantize.hip", "apb_forward.hip", "apb_sparse.hip", "apb_rows.hip",
           "apb_binary_mfma.hip", "apb_binary_mfma_d1.hip", "apb_binary_mfma_d2.hip", "apb_binary_mfma_22i.hip",
           "apb_binary_mfma_22f.hip", "apb_noalloc.hip", "apb_probe.hip", "apb_train.hip"]

# Packed-FP32 VALU forms are disabled on purpose; contraction is off so that every fused
# multiply-add in the kernels is one written explicitly.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd, verbose):
    t0 = time.perf_counter()
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # (the host pass does not know the packed-fp32 feature flag and says so once per file: harmless)
    out = "\n".join(l for l in p.stdout.splitlines() if "is not a recognized feature for this target" not in l)
    if verbose or p.returncode != 0:
        print(f"[{time.perf_counter() - t0:6.1f} s] {' '.join(cmd)}\n{out}", flush=True)
    if p.returncode != 0:
        raise subprocess.CalledProcessError(p.returncode, cmd)


def build(verbose: bool = True, extra_flags=(), force: bool = True, jobs: int = 0) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    headers = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h")) + [__file__]
    newest_header = max(os.path.getmtime(h) for h in headers)
    todo, objs = [], []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ_DIR, s.replace(".hip", ".o"))
        objs.append(obj)
        stale = force or not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), newest_header)
        if stale:
            todo.append([hipcc(), *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                         "-c", src, "-o", obj])
    jobs = jobs or max(1, min(len(os.sched_getaffinity(0)), 16))
    with concurrent.futures.ThreadPoolExecutor(jobs) as pool:
        for f in [pool.submit(_run, c, verbose) for c in todo]:
            f.result()
    if todo or not os.path.exists(LIB):
        _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    build(force="--changed" not in sys.argv[1:], extra_flags=[a for a in sys.argv[1:] if a != "--changed"])
