"""A few latency-bound kernels request a scalar value by hand (an s_load_dword in an inline assembly statement)
long before they need it and wait for it with a second statement (s_waitcnt lgkmcnt(0)) right before the use: the
compiler knows nothing of the load in flight, so the destination register must not be read or written between
the two.  This test compiles those sources to gfx950 assembly and checks exactly that, in every instantiation."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2602_01053_amd", "csrc")
SOURCES = ["lra_generic.hip", "lra_append.hip"]


def _regs(line):
    """Scalar registers a line of assembly names: sN and the members of s[a:b]."""
    out = set(int(m) for m in re.findall(r"\bs(\d+)\b", line))
    for a, b in re.findall(r"\bs\[(\d+):(\d+)\]", line):
        out.update(range(int(a), int(b) + 1))
    return out


def check_asm(text):
    """Returns (hand-issued loads found, list of violations)."""
    found, bad = 0, []
    lines = text.splitlines()
    i = 0
    func = "?"
    while i < len(lines):
        ln = lines[i]
        m = re.match(r"^(_Z\w+):", ln)
        if m:
            func = m.group(1)
        if "#ASMSTART" in ln and i + 1 < len(lines):
            m = re.match(r"\s*s_load_dword s(\d+), s\[(\d+):(\d+)\]", lines[i + 1])
            if m:
                found += 1
                dest = int(m.group(1))
                j = i + 2
                while j < len(lines) and "s_endpgm" not in lines[j]:
                    body = lines[j].split(";")[0]
                    if "s_waitcnt" in body and "lgkmcnt(0)" in body:
                        break
                    if dest in _regs(body):
                        bad.append((func, j + 1, lines[j].strip()))
                        break
                    j += 1
                else:
                    bad.append((func, i + 2, "no wait before the end of the kernel"))
        i += 1
    return found, bad


def test_checker_sees_a_planted_hazard():
    good = "_Zk:\n ;;#ASMSTART\n s_load_dword s5, s[2:3], 0x0\n ;;#ASMEND\n s_add_i32 s6, s7, 1\n s_waitcnt lgkmcnt(0)\n s_add_i32 s5, s5, 1\n s_endpgm\n"
    hazard = good.replace("s_add_i32 s6, s7, 1", "s_add_i32 s6, s5, 1")
    ranged = good.replace("s_add_i32 s6, s7, 1", "s_load_dwordx4 s[4:7], s[0:1], 0x0")
    assert check_asm(good) == (1, [])
    assert check_asm(hazard)[1] and check_asm(ranged)[1]


@pytest.mark.parametrize("src", SOURCES)
def test_hand_issued_scalar_loads_are_not_touched_before_their_wait(src, tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    from paper_2602_01053_amd.build import HIPCC_FLAGS
    out = tmp_path / (src + ".s")
    flags = [f for f in HIPCC_FLAGS if f != "-fPIC"]
    res = subprocess.run([hipcc, *flags, "-S", "--cuda-device-only", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                          os.path.join(CSRC, src), "-o", str(out)], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    found, bad = check_asm(out.read_text())
    assert found > 0, "no hand-issued scalar load found: the checker no longer matches the sources"
    assert not bad, bad[:5]
