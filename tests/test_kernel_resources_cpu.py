"""What the compiler reports for every kernel of the built library (registers, scratch memory, LDS, occupancy):
the build writes the table beside the library, and this test holds it against the figures the design relies on.
Scratch memory in a steady-state loop would be a silent slowdown; a kernel that loses its second wave per SIMD
or grows past the LDS of a compute unit would be one too."""
from __future__ import annotations

import json
import os
import re

import pytest

import paper_2602_01053_amd as lra
from paper_2602_01053_amd import build as lra_build

SCRATCH = "ScratchSize [bytes/lane]"
LDS = "LDS Size [bytes/block]"
OCC = "Occupancy [waves/SIMD]"


@pytest.fixture(scope="module")
def table():
    if not os.path.exists(lra_build.RESOURCES_PATH) or not os.path.exists(lra.binding.LIB_PATH):
        lra_build.build_library()
    with open(lra_build.RESOURCES_PATH) as f:
        doc = json.load(f)
    if doc.get("source_fingerprint") != lra_build.source_fingerprint():  # a table of other sources says nothing
        lra_build.build_library()
        with open(lra_build.RESOURCES_PATH) as f:
            doc = json.load(f)
    assert doc["source_fingerprint"] == lra_build.source_fingerprint()
    return doc["kernels"]


def _args(name: str):
    """Template arguments of a mangled kernel name, as the integers and booleans they are."""
    return [int(v) if t == "i" else bool(int(v)) for t, v in re.findall(r"L([ib])(\d+)E", name)]


def test_every_kernel_is_listed(table):
    names = " ".join(table)
    for kernel in ("decode_stream_kernel", "decode_mfma_kernel", "decode_qt_prepass_kernel", "prefill_mfma_kernel",
                   "complete_rope_keys_kernel", "merge_rows_kernel", "merge_wave_kernel", "merge_kernel",
                   "generic_partial_kernel", "generic_partial_rope_kernel", "append_kernel", "append_finish_kernel",
                   "append_wide_kernel", "append_skinny_kernel", "append_gemv_kernel"):
        assert kernel in names, kernel
    for row in table.values():
        assert row["Dynamic Stack"] == "False"
        assert row[LDS] <= 160 * 1024


# kernels that are allowed scratch memory, with the most each may use (bytes per lane) and why
SCRATCH_ALLOWED = [
    # one accumulator tuple parked between the loop and the store (none inside the loop)
    (r"append_wide_kernel", 136),
    # rotary prefill that completes key tiles itself and writes partial states: loop-invariant addresses
    (r"prefill_mfma_kernelILi\d+ELi\d+ELb[01]ELb0ELb1ELb1ELb0E", 192),
    # rank 64 with a Qt term on paged caches: a few registers over 256
    (r"prefill_mfma_kernelILi128ELi64ELb1ELb1ELb[01]ELb0ELb0E", 16),
    # rotary decode at d = 128, ranks up to 16 and 33..64: a few registers over the file (B_K^T operands of four agent
    # slots stay in registers); up to nine values spilled, five reloads per 32-key step
    (r"decode_mfma_kernelILi128ELi1ELi(32|64)ELb[01]ELb1ELb0ELi(16|64)E", 160),
]


def test_scratch_memory_only_where_listed(table):
    for name, row in table.items():
        if row[SCRATCH] == 0:
            continue
        limits = [cap for pat, cap in SCRATCH_ALLOWED if re.search(pat, name)]
        assert limits, f"{name} uses {row[SCRATCH]} B of scratch memory per lane"
        assert row[SCRATCH] <= max(limits), (name, row[SCRATCH])


def test_headline_kernels(table):
    """The instantiations the headline workloads run: no scratch, the occupancy and LDS their design states."""
    seen = set()
    for name, row in table.items():
        a = _args(name)
        if "decode_stream_kernel" in name:
            # two workgroups' worth of registers are never needed (one workgroup of 512 threads per CU), but no scratch
            assert row[SCRATCH] == 0 and row["AGPRs"] == 0, name
            if a[:3] == [128, 1, 32] and a[3:] == [True, False, False, True]:  # config 2
                assert row["VGPRs"] <= 128 and row[LDS] <= 160 * 1024, (name, row)
                seen.add("cfg2")
        if "merge_rows_kernel" in name or "merge_wave_kernel" in name:
            assert row[SCRATCH] == 0 and row["VGPRs"] <= 128, (name, row)
        if "prefill_mfma_kernel" in name and a == [128, 16, False, True, False, False, False]:  # config 3
            assert row[SCRATCH] == 0 and row[OCC] >= 2 and row[LDS] <= 80 * 1024, (name, row)
            seen.add("cfg3")
        if re.search(r"append_kernelILi128ELb0E", name) or "append_gemv_kernel" in name or "append_finish_kernel" in name:
            assert row[SCRATCH] == 0, name
    assert seen == {"cfg2", "cfg3"}
