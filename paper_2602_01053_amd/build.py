"""Compile the HIP library (and nothing else) for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "liblra_attn.so")

SOURCES = ["lra_plan.cpp", "lra_api.hip", "lra_generic.hip", "lra_decode_mfma.hip", "lra_decode_stream.hip", "lra_prefill_mfma.hip", "lra_append.hip", "lra_probe.hip"]

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
    # packed fp32 instructions are kept out of every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # the LDS transfers set M0 inside their assembly statement and say so in the clobber list
    "-Wno-inline-asm",
]


def source_fingerprint() -> str:
    """Hash (16 hex digits) of everything the library is compiled from: the sources, the headers
    beside them and the public headers.  Measurements kept next to the code (HBM traffic per launch
    from hardware counters) record it, so that a reader can tell whether they were taken on these
    kernels or on earlier ones."""
    import hashlib
    h = hashlib.sha256()
    inc = os.path.join(ROOT, "include")
    files = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith((".hip", ".h", ".cpp"))]
    files += [os.path.join(inc, f) for f in sorted(os.listdir(inc)) if f.endswith(".h")]
    for path in files:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops"
    err = "\n".join(ln for ln in res.stderr.splitlines() if noise not in ln)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}): {' '.join(cmd)}\n{err}")
    if verbose and err.strip():
        print(err)


def build_library(verbose: bool = False) -> str:
    """Compile every source to an object file (in parallel, under _build/) and link the shared library."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    obj_dir = os.path.join(ROOT, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    jobs = []
    for src in SOURCES:
        path = os.path.join(CSRC, src)
        if not os.path.exists(path):
            raise FileNotFoundError(path)
        obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
        if src.endswith(".cpp"):   # host-only C++ (launch planning): no device pass
            jobs.append(([hipcc, "-O2", "-std=c++17", "-fPIC", *inc, "-c", path, "-o", obj], obj))
        else:
            jobs.append(([hipcc, *HIPCC_FLAGS, *inc, "-c", path, "-o", obj], obj))
    with ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 1)) as pool:
        list(pool.map(lambda j: _run(j[0], verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *[o for _, o in jobs], "-o", LIB_PATH], verbose)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
