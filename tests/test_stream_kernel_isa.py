"""Static check of the streaming kernel's generated gfx950 assembly.

The kernel issues its input-fragment loads from inline assembly and waits for
them with hand-counted ``s_waitcnt vmcnt(N)`` so that a wave never waits for
its previous tile's stores.  The compiler does not track those loads, so this
test compiles the source to assembly and verifies, for every instance whose K
loops are compile-time exact:
  * before the first use of a fragment's registers the loop head has executed
    a wait with N <= (fragment loads issued after it) + (stores per tile);
  * between a fragment's load and the end of the loop body nothing reads or
    writes its destination registers (no compiler-inserted copies).
Instances with run-time K guards must use a full ``vmcnt(0)`` wait.
"""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2601_11608_amd", "csrc", "conv_stream.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def vregs(line):
    regs = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", line):
        regs.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", line):
        regs.add(int(m.group(1)))
    return regs


@pytest.fixture(scope="module")
def asm():
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not available")
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "conv_stream.s")
        subprocess.check_call(
            [HIPCC, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-S", "--cuda-device-only", SRC, "-o", out],
            stderr=subprocess.DEVNULL)
        return open(out).read()


def loop_lines(asm, name):
    i = asm.index(name + ":")
    body = asm[i:asm.index("s_endpgm", i)]
    k = body.index("Loop Header")
    return [l.strip() for l in body[k:].splitlines()
            if l.strip() and not l.strip().startswith(";") and not l.strip().startswith(".")]


def test_hand_counted_waits_cover_every_fragment(asm):
    names = sorted(set(re.findall(r"^(_ZN12_GLOBAL__N_118conv_stream_kernelI\S+?):", asm, re.M)))
    assert len(names) >= 40
    checked = 0
    for name in names:
        m = re.search(r"TraitsLi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)ELb([01])ELb([01])E", name)
        nt, khm, ksm, exact = int(m.group(1)), int(m.group(2)), int(m.group(3)), m.group(5) == "1"
        passes = 2 * nt                      # 16-byte store passes per 32-row tile of 32*nt columns
        lines = loop_lines(asm, name)
        loads = [i for i, l in enumerate(lines) if l.startswith("buffer_load_dwordx4")]
        assert len(loads) == khm * ksm, name
        stores_after = sum(1 for l in lines[loads[-1]:] if l.startswith("buffer_store_dwordx4"))
        waits = [int(w) for l in lines for w in re.findall(r"s_waitcnt vmcnt\((\d+)\)", l)]
        if not exact:
            assert waits and all(w == 0 for w in waits), name
            continue
        # the loop text holds the stores that follow the loads, except that the compiler may rotate
        # the last one to the head of the next trip; either way at least passes-1 are visible here
        assert stores_after >= passes - 1, name
        need = {}
        for pos, i in enumerate(loads):
            mm = re.match(r"buffer_load_dwordx4 v\[(\d+):(\d+)\]", lines[i])
            for r in range(int(mm.group(1)), int(mm.group(2)) + 1):
                need[r] = (len(loads) - 1 - pos) + passes
        waited = 10 ** 9
        for l in lines[:loads[0]]:
            w = re.match(r"s_waitcnt vmcnt\((\d+)\)", l)
            if w:
                waited = min(waited, int(w.group(1)))
                continue
            for r in vregs(l):
                assert r not in need or waited <= need[r], "%s: '%s' touches v%d before its load landed" % (name, l, r)
        pending = set()
        for l in lines[loads[0]:]:
            mm = re.match(r"buffer_load_dwordx4 v\[(\d+):(\d+)\]", l)
            if mm:
                pending.update(range(int(mm.group(1)), int(mm.group(2)) + 1))
                continue
            assert not (vregs(l) & pending), "%s: '%s' touches registers of a load in flight" % (name, l)
        checked += 1
    assert checked >= 20
