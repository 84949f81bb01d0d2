"""Static check of the LDS-tiled kernel's generated gfx950 assembly.

The kernel stages its operands with buffer loads that deposit straight into
LDS, issued from inline assembly two K blocks ahead, and publishes each block
with a hand-counted ``s_waitcnt vmcnt(N)`` followed by a barrier.  The compiler
does not track those loads, so this test compiles the source to assembly and
walks every path through each instance's control flow (loop back edges
included, states memoised per block), counting loads in flight: loads complete
in issue order, a wait with count N leaves at most N outstanding.  It verifies
that
  * every load-to-LDS sets M0 in the instruction before it;
  * at every barrier at most one block's worth of loads (the block after the
    one being published) is still in flight;
  * nothing is in flight when LDS is written by ordinary instructions (the
    epilogue reuses the stages), at a global store, or at the end.
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


def explore(lines, name, per_block):
    """Every path through the kernel's control flow; state = number of loads-to-LDS in flight."""
    label_at = {l[:-1]: i for i, l in enumerate(lines) if l.endswith(":")}
    seen, work, ends, barriers = set(), [(0, 0)], 0, 0
    while work:
        pc, n = work.pop()
        while True:
            l = lines[pc]
            if l.endswith(":"):
                if (pc, n) in seen:
                    break
                seen.add((pc, n))
                pc += 1
                continue
            if l == "s_endpgm":
                assert n == 0, "%s: loads still in flight at the end of the kernel" % name
                ends += 1
                break
            b = re.match(r"s_(c?)branch\w* (\.LBB\d+_\d+)$", l)
            if b:
                target = label_at[b.group(2)]
                if b.group(1):
                    work.append((target, n))
                    pc += 1
                else:
                    pc = target
                continue
            if re.match(r"buffer_load_dwordx4 .* lds$", l):
                assert lines[pc - 1].startswith("s_mov_b32 m0,"), "%s: load-to-LDS without its M0 setup" % name
                n += 1
            elif l.startswith("buffer_load") or l.startswith("global_load"):
                pass  # tracked by the compiler (bias); younger loads only make the hand-counted waits stricter
            else:
                w = re.match(r"s_waitcnt .*vmcnt\((\d+)\)", l)
                if w:
                    n = min(n, int(w.group(1)))
                elif l == "s_barrier":
                    assert n <= per_block, "%s: barrier passed with %d loads in flight" % (name, n)
                    barriers += 1
                elif l.startswith("ds_write") or l.startswith("global_store") or l.startswith("buffer_store"):
                    assert n == 0, "%s: '%s' while loads-to-LDS are in flight" % (name, l)
            pc += 1
    assert ends >= 1 and barriers >= 3
    return len(seen)


def loads_per_block(lines):
    n = sum(1 for l in lines if re.match(r"buffer_load_dwordx4 .* lds$", l))
    assert n % 3 == 0, n                 # two blocks in the prologue, one in the loop body
    return n // 3


def test_staging_loads_are_published_with_the_right_counts(asm):
    names = sorted(set(re.findall(r"^(_ZN12_GLOBAL__N_117conv_tiled_kernelI\S+?):", asm, re.M)))
    assert len(names) == 12
    for name in names:
        lines = instructions(asm, name)
        nl = loads_per_block(lines)
        assert nl in (4, 5, 6), (name, nl)
        waits = [int(w) for l in lines for w in re.findall(r"s_waitcnt vmcnt\((\d+)\)$", l)]
        assert 0 in waits and waits.count(nl) >= 2, (name, waits)
        assert explore(lines, name, nl) > 10
        # M0 is written by the inline assembly without the compiler knowing: nothing else may use it
        others = [l for l in lines if re.search(r"\bm0\b", l) and not l.startswith("s_mov_b32 m0,")]
        assert not others, (name, others[:3])


@pytest.mark.parametrize("mutation", ["drop_wait", "weak_wait", "no_drain", "no_m0"])
def test_walker_catches_planted_mistakes(asm, mutation):
    name = sorted(set(re.findall(r"^(_ZN12_GLOBAL__N_117conv_tiled_kernelI\S+?):", asm, re.M)))[0]
    lines = instructions(asm, name)
    nl = loads_per_block(lines)
    idx = [i for i, l in enumerate(lines) if re.match(r"s_waitcnt vmcnt\(%d\)$" % nl, l)]
    drains = [i for i, l in enumerate(lines) if re.match(r"s_waitcnt vmcnt\(0\)$", l)]
    bad = list(lines)
    if mutation == "drop_wait":
        bad[idx[-1]] = "s_nop 0"
    elif mutation == "weak_wait":
        bad[idx[-1]] = "s_waitcnt vmcnt(%d)" % (nl + 1)
    elif mutation == "no_drain":
        for i in drains[1:]:            # keep the one ahead of the prologue
            bad[i] = "s_nop 0"
    else:
        first = next(i for i, l in enumerate(lines) if re.match(r"buffer_load_dwordx4 .* lds$", l))
        bad[first - 1] = "s_nop 0"
    with pytest.raises(AssertionError):
        explore(bad, name, nl)
