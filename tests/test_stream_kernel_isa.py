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
        # 16-byte store passes per 32-row tile of 32*nt columns: 8 elements per piece, 4 for fp32
        passes = (4 if "F32" in name else 2) * nt
        lines = loop_lines(asm, name)
        loads = [i for i, l in enumerate(lines) if re.match(r"buffer_load_dwordx[24] ", l)]   # dwordx2: 8-byte operand chunks
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
            mm = re.match(r"buffer_load_dwordx[24] v\[(\d+):(\d+)\]", lines[i])
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
            mm = re.match(r"buffer_load_dwordx[24] v\[(\d+):(\d+)\]", l)
            if mm:
                pending.update(range(int(mm.group(1)), int(mm.group(2)) + 1))
                continue
            assert not (vregs(l) & pending), "%s: '%s' touches registers of a load in flight" % (name, l)
        checked += 1
    assert checked >= 20


# ---- the same property by walking every path through the control flow -------------------------
# Used for the channels-first streaming kernel, whose loop the compiler rotates (the previous tile's
# stores sit at the top of the loop text), and as a second check of the channels-last one.
NCHW_SRC = os.path.join(ROOT, "paper_2601_11608_amd", "csrc", "conv_stream_nchw.hip")


def compile_to_asm(src):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not available")
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        import sys
        sys.path.insert(0, ROOT)
        from paper_2601_11608_amd.build import device_flags   # the flags the library is built with
        subprocess.check_call(
            [HIPCC, "-O3", "-std=c++17"] + device_flags(src) + ["-S", "--cuda-device-only", src, "-o", out],
            stderr=subprocess.DEVNULL)
        return open(out).read()


def instructions(asm, name):
    i = asm.index(name + ":")
    body = asm[i:asm.index(".Lfunc_end", i)]       # a kernel may have several s_endpgm
    out = []
    for l in body.splitlines()[1:]:
        l = l.split(";")[0].strip()
        if l and (not l.startswith(".") or re.match(r"\.LBB\d+_\d+:", l)):
            out.append(l)
    return out


def walk_paths(lines, name):
    """Loads complete in issue order and a wait with count N leaves at most N vector-memory
    operations outstanding, so a hand-issued load has landed once a wait's count is no larger than
    the number of vector-memory operations issued after it.  State per path: the hand-issued loads
    in flight, each with its destination registers and that number.  Fails if anything touches the
    registers of a load that has not landed."""
    label_at = {l[:-1]: i for i, l in enumerate(lines) if l.endswith(":")}
    seen, work, ends, landed_by_count = set(), [(0, ())], 0, 0
    while work:
        pc, state = work.pop()
        while True:
            l = lines[pc]
            if l.endswith(":"):
                if (pc, state) in seen:
                    break
                seen.add((pc, state))
                assert len(seen) < 200000, name
                pc += 1
                continue
            if l == "s_endpgm":
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
            w = re.search(r"s_waitcnt.*vmcnt\((\d+)\)", l)
            if w:
                n = int(w.group(1))
                if n > 0:
                    landed_by_count += sum(1 for regs, after in state if after >= n)
                state = tuple((regs, after) for regs, after in state if after < n)
                pc += 1
                continue
            touched = vregs(l)
            m = re.match(r"buffer_load_dwordx[24] v\[(\d+):(\d+)\]", l)
            # a zero-extended 2-byte load into a register of its own (the channels-first input gather)
            h = re.match(r"buffer_load_ushort v(\d+),", l)
            for regs, _ in state:
                assert not (touched & regs), "%s: '%s' touches registers of a load in flight" % (name, l)
            if re.match(r"(buffer|global|flat|scratch)_(load|store|atomic)", l):
                state = tuple((regs, min(after + 1, 64)) for regs, after in state)
            if m:
                state = state + ((frozenset(range(int(m.group(1)), int(m.group(2)) + 1)), 0),)
            if h:
                state = state + ((frozenset([int(h.group(1))]), 0),)
            pc += 1
    assert ends >= 1
    return landed_by_count


@pytest.fixture(scope="module")
def nchw_asm():
    return compile_to_asm(NCHW_SRC)


def test_channels_first_kernel_waits(nchw_asm):
    names = sorted(set(re.findall(r"^(_ZN12_GLOBAL__N_123conv_stream_nchw_kernelI\S+?):", nchw_asm, re.M)))
    # two dtypes x two (KH, K-step) shapes x exact/guarded x ReLU x (width fold; height fold in blocks of two, four or eight tiles; each also with a channels-first input)
    assert len(names) == 128
    for name in names:
        exact = re.search(r"TraitsLi\d+ELi\d+ELb([01])ELb[01]ELb[01]ELb[01]ELi\d+ELb[01]E", name).group(1) == "1"
        lines = instructions(nchw_asm, name)
        partial = walk_paths(lines, name)
        counts = [int(w) for l in lines for w in re.findall(r"s_waitcnt.*vmcnt\((\d+)\)", l)]
        # the last template argument: width fold with the channels-first input staged through LDS
        staged = re.search(r"TraitsLi\d+ELi\d+ELb[01]ELb[01]ELb[01]ELb[01]ELi\d+ELb([01])E", name).group(1) == "1"
        if exact or staged:
            # the stores of the previous tile stay in flight: some waits leave 4 or more outstanding
            # (a staged instance waits that way for its piece of the input, guarded K loop or not)
            assert partial > 0 and max(counts) >= 4, name
        else:
            assert partial == 0, name


def test_channels_last_kernel_waits_by_path_walk(asm):
    names = sorted(set(re.findall(r"^(_ZN12_GLOBAL__N_118conv_stream_kernelI\S+?):", asm, re.M)))
    for name in names:
        walk_paths(instructions(asm, name), name)


@pytest.mark.parametrize("mutation", ["weak_wait", "drop_store"])
def test_path_walk_catches_planted_mistakes(nchw_asm, mutation):
    name = next(n for n in sorted(set(re.findall(r"^(_ZN12_GLOBAL__N_123conv_stream_nchw_kernelI\S+?):", nchw_asm, re.M)))
                if "Li3ELi1ELb1ELb0ELb0ELb0ELi0ELb0E" in n)
    lines = instructions(nchw_asm, name)
    walk_paths(lines, name)
    bad = list(lines)
    if mutation == "weak_wait":
        # one more operation allowed in flight than there are behind the fragment's load
        i = max(i for i, l in enumerate(bad) if re.match(r"s_waitcnt vmcnt\(4\)$", l))
        bad[i] = "s_waitcnt vmcnt(5)"
    else:
        # one store fewer between the loads and the wait: the count no longer covers the load
        i = max(i for i, l in enumerate(bad) if l.startswith("buffer_store_dwordx4"))
        bad[i] = "s_nop 0"
    with pytest.raises(AssertionError):
        walk_paths(bad, name)


# ---- the LDS-staged dense-walk kernel: loads that deposit into LDS, counted by hand -------------
LDS_SRC = os.path.join(ROOT, "paper_2601_11608_amd", "csrc", "conv_stream_lds.hip")


def walk_lds_loads(lines, name, per_tile):
    """Every path through the kernel.  State: for each load-to-LDS in flight, the number of
    vector-memory operations issued after it (loads complete in issue order; a wait with count N
    leaves at most N operations outstanding).  Checks that every such load sets M0 in the
    instruction before it, that at every barrier only the loads of one tile (the one after the
    tile being published) can still be in flight, and that none is in flight at the end."""
    label_at = {l[:-1]: i for i, l in enumerate(lines) if l.endswith(":")}
    seen, work, ends, barriers = set(), [(0, ())], 0, 0
    while work:
        pc, state = work.pop()
        while True:
            l = lines[pc]
            if l.endswith(":"):
                if (pc, state) in seen:
                    break
                seen.add((pc, state))
                assert len(seen) < 200000, name
                pc += 1
                continue
            if l == "s_endpgm":
                assert not state, "%s: loads-to-LDS in flight at the end of the kernel" % name
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
            w = re.search(r"s_waitcnt.*vmcnt\((\d+)\)", l)
            if w:
                state = tuple(a for a in state if a < int(w.group(1)))
            elif l == "s_barrier":
                assert len(state) <= per_tile, "%s: barrier passed with %d loads-to-LDS in flight" % (name, len(state))
                barriers += 1
            elif re.match(r"(buffer|global|flat|scratch)_(load|store|atomic)", l):
                state = tuple(min(a + 1, 64) for a in state)
                if re.match(r"buffer_load_dwordx4 .* lds$", l):
                    assert lines[pc - 1].startswith("s_mov_b32 m0,"), "%s: load-to-LDS without its M0 setup" % name
                    state = state + (0,)
            pc += 1
    assert ends >= 1 and barriers >= 2
    return len(seen)


@pytest.fixture(scope="module")
def lds_asm():
    return compile_to_asm(LDS_SRC)


def lds_kernel_names(asm):
    return sorted(set(re.findall(r"^(_ZN12_GLOBAL__N_122conv_stream_lds_kernelI\S+?):", asm, re.M)))


def test_staged_input_kernel_waits(lds_asm):
    names = lds_kernel_names(lds_asm)
    assert len(names) == 4
    for name in names:
        lines = instructions(lds_asm, name)
        n_loads = sum(1 for l in lines if re.match(r"buffer_load_dwordx4 .* lds$", l))
        assert n_loads % 7 == 0 and n_loads >= 28, (name, n_loads)   # 7 per wave and tile: two tiles in the prologue, one per loop body
        assert walk_lds_loads(lines, name, 7) > 10
        others = [l for l in lines if re.search(r"\bm0\b", l) and not l.startswith("s_mov_b32 m0,")]
        assert not others, (name, others[:3])        # M0 is written behind the compiler's back: nothing else may use it


def test_staged_input_kernel_keeps_accumulators_where_the_epilogue_reads_them(lds_asm):
    """Built with the library's flags, the filter fragments sit in AGPRs and the MFMA results in VGPRs:
    the tile loop copies nothing between the two halves of the register file."""
    for name in lds_kernel_names(lds_asm):
        i = lds_asm.index(name + ":")
        body = lds_asm[i:lds_asm.index(".Lfunc_end", i)]
        loop = body[body.index("Loop Header"):]
        assert "v_accvgpr" not in loop, name
        assert re.search(r"v_mfma_f32_32x32x16_\w+ v\[\d+:\d+\], a\[\d+:\d+\], v\[", loop), name


@pytest.mark.parametrize("mutation", ["weak_wait", "drop_store", "no_drain", "no_m0"])
def test_staged_input_walker_catches_planted_mistakes(lds_asm, mutation):
    name = lds_kernel_names(lds_asm)[0]
    lines = instructions(lds_asm, name)
    walk_lds_loads(lines, name, 7)
    bad = list(lines)
    if mutation == "weak_wait":
        for i, l in enumerate(bad):
            if re.match(r"s_waitcnt vmcnt\(11\)$", l):
                bad[i] = "s_waitcnt vmcnt(12)"
    elif mutation == "drop_store":
        for i, l in enumerate(bad):          # one store fewer per tile: the count no longer covers the tile's loads
            if l.startswith("buffer_store_dwordx4") and "nt" in l:
                bad[i] = "s_nop 0"
                break
        # the loop bodies hold the other stores; drop one in each run of four
        runs = [i for i, l in enumerate(bad) if l.startswith("buffer_store_dwordx4")]
        for i in runs[::4]:
            bad[i] = "s_nop 0"
    elif mutation == "no_drain":
        drains = [i for i, l in enumerate(bad) if re.match(r"s_waitcnt vmcnt\(0\)$", l)]
        for i in drains[1:]:
            bad[i] = "s_nop 0"
    else:
        first = next(i for i, l in enumerate(bad) if re.match(r"buffer_load_dwordx4 .* lds$", l))
        bad[first - 1] = "s_nop 0"
    with pytest.raises(AssertionError):
        walk_lds_loads(bad, name, 7)
