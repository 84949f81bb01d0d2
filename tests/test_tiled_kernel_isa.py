"""Static check of the LDS-tiled kernel's generated gfx950 assembly.

The kernel issues its staging loads from inline assembly (two register sets,
software-pipelined two K blocks ahead) and waits for them with explicit
``s_waitcnt vmcnt(N)``.  The compiler does not track those loads, so this test
compiles the source to assembly and walks every instance's K loop as the
hardware would retire it: loads complete in issue order, a wait with count N
retires all but the N newest.  Along every path through the kernel's control
flow (loop back edges included, states memoised per block) it verifies that
  * no instruction reads or writes the destination registers of a load that
    is still in flight (in particular no compiler-inserted copy ahead of the
    wait);
  * nothing is in flight when a store is issued or the kernel ends (the drain).
A second test plants mistakes in the assembly text and expects the walker to object.
"""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2601_11608_amd", "csrc", "conv_tiled.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def vregs(text):
    regs = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", text):
        regs.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", text):
        regs.add(int(m.group(1)))
    return regs


@pytest.fixture(scope="module")
def asm():
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not available")
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "conv_tiled.s")
        subprocess.check_call(
            [HIPCC, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-S", "--cuda-device-only", SRC, "-o", out],
            stderr=subprocess.DEVNULL)
        return open(out).read()


def instructions(asm, name):
    i = asm.index(name + ":")
    body = asm[i:asm.index("s_endpgm", i)] + "s_endpgm\n"
    out = []
    for l in body.splitlines()[1:]:
        l = l.split(";")[0].strip()
        if l and (not l.startswith(".") or re.match(r"\.LBB\d+_\d+:", l)):
            out.append(l)
    return out


def step(l, name, in_flight):
    """Apply one instruction to the FIFO of loads in flight (tuple of frozensets of registers)."""
    pending = frozenset().union(*in_flight) if in_flight else frozenset()
    m = re.match(r"buffer_load_dwordx4 v\[(\d+):(\d+)\]", l)
    if m:
        dst = frozenset(range(int(m.group(1)), int(m.group(2)) + 1))
        addr = vregs(l.split(",", 1)[1])
        assert not (addr & pending), "%s: '%s' takes its address from a register in flight" % (name, l)
        assert not (dst & pending), "%s: '%s' overwrites a register in flight" % (name, l)
        return in_flight + (dst,)
    w = re.match(r"s_waitcnt .*vmcnt\((\d+)\)", l)
    if w:
        n = int(w.group(1))
        return in_flight[len(in_flight) - n:] if n < len(in_flight) else in_flight
    if l.startswith("s_waitcnt"):
        return in_flight
    assert not (vregs(l) & pending), "%s: '%s' touches registers of a load in flight" % (name, l)
    return in_flight


def explore(lines, name):
    """Every path through the kernel's control flow, loads retiring in issue order."""
    label_at = {l[:-1]: i for i, l in enumerate(lines) if l.endswith(":")}
    seen, work, ends = set(), [(0, ())], 0
    while work:
        pc, state = work.pop()
        while True:
            l = lines[pc]
            if l.endswith(":"):
                if (pc, state) in seen:
                    break
                seen.add((pc, state))
                pc += 1
                continue
            if l == "s_endpgm":
                assert state == (), "%s: loads still in flight at the end of the kernel" % name
                ends += 1
                break
            b = re.match(r"s_(c?)branch\w* (\.LBB\d+_\d+)$", l)
            if b:
                target = label_at[b.group(2)]
                if b.group(1):
                    work.append((target, state))
                    pc += 1
                else:
                    pc = target
                continue
            if l.startswith("global_store") or l.startswith("buffer_store"):
                assert state == (), "%s: a store is issued while staging loads are in flight" % name
            state = step(l, name, state)
            pc += 1
    assert ends >= 1
    return len(seen)


def test_staging_loads_are_never_touched_in_flight(asm):
    names = sorted(set(re.findall(r"^(_ZN12_GLOBAL__N_117conv_tiled_kernelI\S+?):", asm, re.M)))
    assert len(names) == 8
    for name in names:
        lines = instructions(asm, name)
        n_loads = sum(1 for l in lines if l.startswith("buffer_load_dwordx4"))
        assert n_loads in (16, 24), (name, n_loads)      # prologue + unrolled loop: four sets of NL = 4 or 6
        waits = [int(w) for l in lines for w in re.findall(r"s_waitcnt vmcnt\((\d+)\)$", l)]
        assert 0 in waits and any(0 < w <= n_loads // 4 for w in waits), (name, waits)
        assert explore(lines, name) > 10


@pytest.mark.parametrize("mutation", ["drop_wait", "weak_wait", "no_drain"])
def test_walker_catches_planted_mistakes(asm, mutation):
    name = sorted(set(re.findall(r"^(_ZN12_GLOBAL__N_117conv_tiled_kernelI\S+?):", asm, re.M)))[0]
    lines = instructions(asm, name)
    nl = sum(1 for l in lines if l.startswith("buffer_load_dwordx4")) // 4
    idx = [i for i, l in enumerate(lines) if re.match(r"s_waitcnt vmcnt\([1-9]\)$", l)]
    drains = [i for i, l in enumerate(lines) if re.match(r"s_waitcnt vmcnt\(0\)$", l)]
    bad = list(lines)
    if mutation == "drop_wait":
        bad[idx[-1]] = "s_nop 0"
    elif mutation == "weak_wait":
        bad[idx[-1]] = "s_waitcnt vmcnt(%d)" % (int(re.search(r"\((\d+)\)", lines[idx[-1]]).group(1)) + 1)
    else:
        for i in drains[1:]:            # keep the one ahead of the prologue
            bad[i] = "s_nop 0"
    with pytest.raises(AssertionError):
        explore(bad, name)
