"""Compile the HIP library (and nothing else) for gfx950, in-tree."""
from __future__ import annotations

import os
import re
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "liblra_attn.so")
# what the compiler reports per kernel (registers, scratch, LDS, occupancy), written by every build
RESOURCES_PATH = os.path.join(PKG_DIR, "kernel_resources.json")

SOURCES = ["lra_plan.cpp", "lra_api.hip", "lra_generic.hip", "lra_decode_mfma.hip", "lra_decode_stream.hip", "lra_prefill_mfma.hip", "lra_append.hip", "lra_probe.hip"]

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
    # packed fp32 instructions are kept out of every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # the LDS transfers set M0 inside their assembly statement and say so in the clobber list
    "-Wno-inline-asm",
]
# (device pass only) one remark block per kernel with its register, scratch and LDS use
RESOURCE_REMARKS = "-Rpass-analysis=kernel-resource-usage"


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


def _parse_resource_remarks(stderr: str) -> dict:
    """{mangled kernel name: {"VGPRs": .., "AGPRs": .., "ScratchSize [bytes/lane]": .., ...}} from the
    compiler's kernel-resource-usage remarks."""
    out, cur = {}, None
    for ln in stderr.splitlines():
        if "[-Rpass-analysis=kernel-resource-usage]" not in ln:
            continue
        m = re.search(r"remark:\s+Function Name: (\S+)", ln)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([^:]+): (\S+) \[-Rpass", ln)
        if m and cur is not None:
            v = m.group(2)
            cur[m.group(1).strip()] = int(v) if v.isdigit() else v
    return out


def _run(cmd, verbose):
    """Runs one compiler command; returns the kernel resource table its remarks hold (empty for host code)."""
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    remarks, rest, skip = [], [], 0
    for ln in res.stderr.splitlines():
        if "[-Rpass-analysis=kernel-resource-usage]" in ln:
            remarks.append(ln)
            skip = 2 if "Function Name" in ln else 0  # (the first remark of a kernel is followed by its source line and a caret)
        elif skip > 0 and re.match(r"^\s+(\d+ \||\|)", ln):
            skip -= 1
        elif "packed-fp32-ops" not in ln:
            rest.append(ln)
    err = "\n".join(rest)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}): {' '.join(cmd)}\n{err}")
    if verbose and err.strip():
        print(err)
    return _parse_resource_remarks("\n".join(remarks))


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
            jobs.append(([hipcc, *HIPCC_FLAGS, RESOURCE_REMARKS, *inc, "-c", path, "-o", obj], obj))
    with ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 1)) as pool:
        tables = list(pool.map(lambda j: _run(j[0], verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *[o for _, o in jobs], "-o", LIB_PATH], verbose)
    import json
    resources = {}
    for (cmd, _), table in zip(jobs, tables):
        for name, row in table.items():
            resources[name] = dict(row, source=os.path.basename(cmd[-3]))
    with open(RESOURCES_PATH, "w") as f:
        json.dump({"source_fingerprint": source_fingerprint(), "kernels": resources}, f, indent=0, sort_keys=True)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
