"""Build libprac.so (HIP, gfx950) in-tree with hipcc.

Usage: python -m paper_2602_23111_amd.build [--incremental]

Every source is compiled to an object file under _build/ (in parallel), then linked.
`incremental=True` skips objects that are newer than their source and the headers.
"""
from __future__ import annotations

import glob
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libprac.so")
SOURCES = ["prac_api.hip", "gemm_bf16.hip", "hot_kernels.hip", "ws_kernels.hip", "gemm_generic.hip",
           "misc_kernels.hip", "fit_basis.hip"]
NOISE = "is not a recognized feature for this target"


def _flags() -> list[str]:
    return ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-I" + os.path.join(ROOT, "include"), "-I" + CSRC] + os.environ.get("PRAC_EXTRA_HIPCC_FLAGS", "").split()


def _run(cmd: list[str]) -> str:
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    return err


def build(verbose: bool = False, incremental: bool = False) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    os.makedirs(OBJ, exist_ok=True)
    headers = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)
    jobs = []
    objs = []
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(OBJ, os.path.splitext(s)[0] + ".o")
        objs.append(obj)
        fresh = (incremental and os.path.exists(obj)
                 and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header))
        if not fresh:
            jobs.append([hipcc] + _flags() + ["-c", "-o", obj, src])
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as pool:
        msgs = list(pool.map(_run, jobs))
    msgs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs))
    if verbose:
        text = "\n".join(m for m in msgs if m.strip())
        if text:
            print(text, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, incremental="--incremental" in sys.argv))
