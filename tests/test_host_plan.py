"""Host-side checks that need no GPU: the C-ABI library loads and exports
every declared symbol, the plan's closed forms agree with the oracle's (which
are pinned by enumeration), error paths, and struct layout."""
import ctypes
import math
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "foldconv.h")


@pytest.fixture(scope="module")
def fc():
    import paper_2601_11608_amd as fc

    if not os.path.exists(fc.library_path()):
        from paper_2601_11608_amd import build

        build.build()
    fc.load_library()
    return fc


def declared_functions():
    text = open(HEADER).read()
    return re.findall(r"FOLDCONV_API\s+[\w\s\*]+?\b(\w+)\s*\(", text)


def test_library_exports_every_declared_symbol(fc):
    names = declared_functions()
    assert set(names) >= {"foldconv_plan", "foldconv_plan_query", "foldconv_plan_destroy", "foldconv_expand_filter",
                          "foldconv_fold_input", "foldconv_unfold_output", "foldconv_pack_filter",
                          "foldconv_forward", "conv_padded_forward", "foldconv_strerror"}
    lib = ctypes.CDLL(fc.library_path())
    for n in names:
        assert getattr(lib, n) is not None, n
    # and the binding offers each of them under the same name
    for n in names:
        assert hasattr(fc, n), n


def test_no_internal_symbols_leak(fc):
    out = subprocess.check_output(["nm", "-D", "--defined-only", fc.library_path()], text=True)
    exported = {l.split()[-1] for l in out.splitlines() if " T " in l}
    assert exported == set(declared_functions())


def test_shapes_struct_layout_matches_c(fc):
    from paper_2601_11608_amd.binding import Shapes

    src = '#include <stdio.h>\n#include <stddef.h>\n#include "foldconv.h"\nint main(){printf("%zu %zu %zu\\n", sizeof(foldconv_shapes_t), offsetof(foldconv_shapes_t, gemm_M), offsetof(foldconv_shapes_t, useful_flops));return 0;}\n'
    with tempfile.TemporaryDirectory() as d:
        c = os.path.join(d, "s.c")
        open(c, "w").write(src)
        exe = os.path.join(d, "s")
        subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), c, "-o", exe])
        size, off_m, off_f = map(int, subprocess.check_output([exe], text=True).split())
    assert ctypes.sizeof(Shapes) == size
    assert Shapes.gemm_M.offset == off_m
    assert Shapes.useful_flops.offset == off_f


PLAN_CASES = [
    # N,H,W,C,Co,KH,KW,pad,F
    (1, 32, 32, 3, 16, 3, 3, 1, 8),
    (64, 224, 224, 3, 64, 3, 3, 1, 16),
    (32, 112, 112, 12, 48, 3, 3, 1, 4),
    (16, 1, 16000, 1, 64, 1, 9, 4, 32),
    (32, 112, 112, 132, 256, 3, 3, 1, 4),
    (1, 32, 64, 1, 1, 5, 1, 0, 8),
    (1, 6, 12, 2, 3, 3, 3, 0, 4),
    (1, 4, 12, 2, 2, 2, 4, 2, 4),
    (2, 5, 7, 3, 3, 3, 3, 1, 1),
]


@pytest.mark.parametrize("N,H,W,C,Co,KH,KW,pad,F", PLAN_CASES)
def test_plan_closed_forms_match_oracle(fc, oracle, N, H, W, C, Co, KH, KW, pad, F):
    p = fc.foldconv_plan(N, H, W, C, Co, KH, KW, pad, F, "float16")
    s = p.shapes
    ph, pw = oracle.axis_pads(KH, KW, pad)
    assert (s.pad_h, s.pad_w) == (ph, pw)
    sh = oracle.folded_shapes(W, KW, pw, F)
    assert (s.W_fold, s.d_min, s.d_max, s.KW_fold) == (sh["Wf"], sh["d_min"], sh["d_max"], sh["KWf"])
    assert (s.W_out, s.W_out_fold) == (sh["W_out"], sh["Wf_out"])
    assert (s.pad_left_fold, s.pad_right_fold) == (sh["pad_left_f"], sh["pad_right_f"])
    assert s.H_out == H + 2 * ph - KH + 1
    assert (s.C_fold, s.Co_fold) == (F * C, F * Co)
    assert s.gemm_M == N * s.H_out * s.W_out_fold and s.gemm_N == F * Co and s.gemm_K == KH * s.KW_fold * F * C
    assert s.w_exp_bytes == s.gemm_K * s.gemm_N * 2
    assert s.x_bytes == N * H * W * C * 2 and s.y_bytes == N * s.H_out * s.W_out * Co * 2
    assert s.y_fold_bytes == s.gemm_M * s.gemm_N * 2
    assert s.unfold_is_alias == int(s.W_out == F * s.W_out_fold)
    assert s.useful_flops == 2.0 * N * s.H_out * s.W_out * Co * KH * KW * C
    assert s.C_pad % 8 == 0 and 0 <= s.C_pad - C < 8
    assert s.issued_flops_band <= s.issued_flops_dense
    assert s.issued_flops_band >= s.useful_flops * 0.999
    p.destroy()


def test_static_scratch_limit_is_checked_before_any_gpu_call(fc):
    """foldconv_forward_static: a plan whose packed filter exceeds the library's static array is
    refused with its own status (no GPU is needed to find that out), bad flags and plans likewise."""
    lib = fc.load_library()
    big = fc.foldconv_plan(1, 8, 64, 132, 256, 3, 3, 1, 16, "float16")
    assert big.shapes.workspace_bytes > fc.STATIC_SCRATCH_BYTES
    assert lib.foldconv_forward_static(big.handle, None, None, None, None, 0, None) == -6
    assert "scratch" in fc.foldconv_strerror(-6)
    ok = fc.foldconv_plan(1, 8, 64, 3, 64, 3, 3, 1, 16, "float16")
    assert 0 < ok.shapes.workspace_bytes <= fc.STATIC_SCRATCH_BYTES
    for flag in (fc.FLAG_FILTER_PACKED, fc.FLAG_FILTER_COMPACT):
        assert lib.foldconv_forward_static(ok.handle, None, None, None, None, flag, None) == -1
    assert lib.foldconv_forward_static(None, None, None, None, None, 0, None) == -1
    header = open(HEADER).read()
    assert int(re.search(r"FOLDCONV_STATIC_SCRATCH_BYTES \((\d+)u << (\d+)\)", header).group(1)) << 20 == fc.STATIC_SCRATCH_BYTES


def test_static_scratch_array_is_a_global_symbol_of_the_device_code():
    """hipGetSymbolAddress finds a device variable by name in the code object: the static array behind
    foldconv_forward_static must come out of the device compilation as a global, 256-byte aligned
    object of the declared size (a local symbol makes the runtime's lookup fail at the first call)."""
    src = os.path.join(ROOT, "paper_2601_11608_amd", "csrc", "static_scratch.hip")
    with tempfile.TemporaryDirectory() as d:
        asm = os.path.join(d, "s.s")
        subprocess.check_call(["/opt/rocm/bin/hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "--cuda-device-only",
                               "-S", src, "-o", asm], stderr=subprocess.DEVNULL)
        text = open(asm).read()
    assert re.search(r"\.globl\s+_ZL7scratch\b", text)
    assert not re.search(r"\.local\s+_ZL7scratch\b", text)
    assert re.search(r"\.size\s+_ZL7scratch, %d\b" % (16 << 20), text)
    assert re.search(r"\.p2align\s+8", text)


def test_prepared_filter_flags_need_a_workspace_the_plan_wrote(fc):
    """FILTER_PACKED / FILTER_COMPACT on a workspace this plan never packed into, and flags the zero-padded
    reference path does not honour, are refused before anything is launched (pointers are never touched)."""
    lib = fc.load_library()
    p = fc.foldconv_plan(2, 8, 64, 3, 64, 3, 3, 1, 16, "float16")
    s = p.shapes
    fake = ctypes.c_void_p(0x7f0000000000)          # aligned, never dereferenced on the host
    big = ctypes.c_size_t(1 << 30)
    assert lib.foldconv_forward(p.handle, fake, fake, None, fake, fake, big, fc.FLAG_FILTER_PACKED, None) == -4
    assert lib.foldconv_forward(p.handle, fake, None, None, fake, fake, big, fc.FLAG_FILTER_COMPACT, None) == -4
    assert lib.conv_padded_forward(p.handle, fake, fake, None, fake, fake, big, fc.FLAG_FILTER_PACKED, None) == -4
    for flag in (fc.FLAG_DENSE_K, fc.FLAG_KEEP_FOLDED, fc.FLAG_FILTER_COMPACT, fc.FLAG_OUT_NCHW, 1 << 20):
        assert lib.conv_padded_forward(p.handle, fake, fake, None, fake, fake, big, flag, None) == -1, flag
    assert s.workspace_bytes > 0


def test_headline_layer_numbers(fc):
    """Sizes of the 224x224 C_in = 3 first layer, F = 16."""
    s = fc.foldconv_plan(64, 224, 224, 3, 64, 3, 3, 1, 16, "float16").shapes
    assert (s.W_fold, s.C_fold, s.Co_fold, s.KW_fold) == (14, 48, 1024, 3)
    assert (s.gemm_M, s.gemm_N, s.gemm_K) == (200704, 1024, 432)
    assert s.y_bytes == 411041792 and s.unfold_is_alias == 1
    assert abs(s.useful_flops - 11.098e9) < 1e7
    assert abs(s.issued_flops_dense - 177.57e9) < 1e8


def test_fused_channels_first_output_is_reported_in_the_plan(fc):
    """shapes.out_nchw_fused: width-folded 16-bit plans whose slots tile whole 16-byte pieces of y."""
    import torch

    def fused(*a, axis=None, dt=torch.float16):
        return fc.foldconv_plan_nchw(*a, fc.FOLD_W if axis is None else axis, dt).shapes.out_nchw_fused

    assert fused(64, 3, 224, 224, 64, 3, 3, 1, 16) == 1                      # the headline layer
    assert fc.foldconv_plan(64, 224, 224, 3, 64, 3, 3, 1, 16, "float16").shapes.out_nchw_fused == 1
    assert fused(64, 3, 224, 224, 64, 3, 3, 1, 16, dt=torch.bfloat16) == 1
    assert fused(64, 3, 224, 224, 64, 3, 3, 1, 16, dt=torch.float32) == 0    # 16-bit types only
    assert fused(64, 3, 224, 224, 64, 3, 3, 1, 16, axis=fc.FOLD_H) == 1      # height fold: pieces run across the plan's rows
    assert fused(64, 3, 224, 220, 64, 3, 3, 1, 16, axis=fc.FOLD_H) == 0      # ... which needs W_out in multiples of 8
    assert fused(64, 3, 224, 224, 64, 3, 3, 1, 4) == 0                       # F not a multiple of 8
    assert fused(64, 3, 224, 224, 64, 3, 3, 1, 32) == 0                      # F*C_out = 2048 > 1024
    assert fused(64, 3, 224, 224, 64, 3, 3, 0, 16) == 0                      # W_out = 222 is not F*W'_out
    assert fused(8, 132, 112, 112, 64, 3, 3, 1, 8) == 0                      # large K: the tiled kernel


def test_plan_errors(fc):
    with pytest.raises(fc.FoldconvError) as e:
        fc.foldconv_plan(1, 8, 10, 3, 4, 3, 3, 1, 4, "float16")
    assert e.value.status == -2                      # Algorithm 1 guard: W mod F != 0
    for bad in [(0, 8, 8, 3, 4, 3, 3, 1, 4), (1, 8, 8, 0, 4, 3, 3, 1, 4), (1, 8, 8, 3, 4, 3, 3, -1, 4),
                (1, 8, 8, 3, 4, 3, 3, 1, 0)]:
        with pytest.raises(fc.FoldconvError) as e:
            fc.foldconv_plan(*bad, "float16")
        assert e.value.status == -1
    with pytest.raises(fc.FoldconvError) as e:
        fc.foldconv_plan(1, 2, 8, 3, 4, 5, 3, 0, 4, "float16")   # VALID kernel taller than the image
    assert e.value.status == -3
    lib = fc.load_library()
    assert lib.foldconv_plan(1, 8, 8, 3, 4, 3, 3, 1, 4, 7, ctypes.byref(ctypes.c_void_p())) == -1   # unknown dtype
    assert lib.foldconv_plan(1, 8, 8, 3, 4, 3, 3, 1, 4, 1, None) == -1
    assert lib.foldconv_plan_query(None, None) == -1
    lib.foldconv_plan_destroy(None)
    for code in range(-6, 1):
        assert isinstance(fc.foldconv_strerror(code), str) and fc.foldconv_strerror(code)


def test_null_pointer_calls_are_rejected_without_gpu(fc):
    """Argument checks come before any HIP call, so they can run on a CPU-only host."""
    lib = fc.load_library()
    p = fc.foldconv_plan(1, 8, 8, 3, 4, 3, 3, 1, 4, "float16")
    h = p.handle
    assert lib.foldconv_expand_filter(h, None, None, None) == -1
    assert lib.foldconv_fold_input(h, None, None, None) == -1
    assert lib.foldconv_unfold_output(h, None, None, None) == -1
    assert lib.foldconv_forward(h, None, None, None, None, None, 0, 0, None) == -1
    assert lib.conv_padded_forward(h, None, None, None, None, None, 0, 0, None) == -1
    assert lib.foldconv_forward(h, 256, 512, None, 1024, None, 0, 1 << 20, None) == -1     # unknown flag
    assert lib.conv_padded_forward(h, 256, 512, None, 1024, None, 0, 0, None) == -4        # workspace missing
    assert lib.foldconv_pack_filter_compact(h, None, 256, 1 << 20, None) == -1
    assert lib.foldconv_pack_filter_compact(h, 512, None, 0, None) == -4                   # workspace missing
    assert lib.foldconv_forward(h, 256, None, None, 1024, None, 0, 16, None) == -4         # compact filter missing
    assert lib.foldconv_forward(h, 256, None, None, 1024, None, 0, 0, None) == -1          # no filter at all
    assert lib.foldconv_fold_input(h, 4096, 4096, None) == 0                               # alias: nothing to do
    assert lib.foldconv_fold_input(h, 4096, 4096 + 16, None) == -1                         # partial overlap


def test_compact_filter_size(fc):
    """Compact storage keeps 8/gcd(C_in,8) zero-padded copies of the KW*C_in x C_out tap matrix per
    kh in 16-byte chunks of 8 rows: close to KW/(KW'*F) of the expanded filter (the density of the
    paper's block structure) once rounding to chunks is small."""
    from paper_2601_11608_amd import workloads as wl

    for name in ("c2", "c3", "c4", "c5"):
        for l in wl.CONFIGS[name]:
            s = fc.foldconv_plan(*l.plan_args(), wl.DTYPES[l.dtype]).shapes
            g8 = math.gcd(l.C_in, 8)
            chunks = (8 - g8 + l.KW * l.C_in + 7) // 8
            want = (8 // g8) * l.KH * chunks * l.C_out * 16
            assert s.filter_compact_bytes == (want + 255) // 256 * 256
            assert s.filter_compact_bytes < s.w_exp_bytes / 3
    s = fc.foldconv_plan(64, 224, 224, 3, 64, 3, 3, 1, 16, "float16").shapes
    assert (s.w_exp_bytes, s.filter_compact_bytes) == (884736, 49152)
    # fp32 on the streaming kernel.  A small layer: chunks of 4 rows (16 bytes), 4/gcd(C_in,4) copies.  A large
    # layer with C_in = 3 (bound by its MFMAs): chunks of 2 rows (8 bytes, fewer structural zeros walked),
    # 2/gcd(C_in,2) copies.  C_in = 12: chunks of 4 rows, one copy
    s = fc.foldconv_plan(1, 32, 32, 3, 16, 3, 3, 1, 8, "float32").shapes
    assert s.conv_kernel == 2 and s.filter_compact_bytes == (4 * 3 * ((4 - 1 + 9 + 3) // 4) * 16 * 16 + 255) // 256 * 256
    s = fc.foldconv_plan(64, 224, 224, 3, 64, 3, 3, 1, 16, "float32").shapes
    assert s.conv_kernel == 2 and s.filter_compact_bytes == (2 * 3 * ((2 - 1 + 9 + 1) // 2) * 64 * 8 + 255) // 256 * 256
    s = fc.foldconv_plan(32, 112, 112, 12, 48, 3, 3, 1, 4, "float32").shapes
    assert s.conv_kernel == 2 and s.filter_compact_bytes == (1 * 3 * ((4 - 4 + 36 + 3) // 4) * 48 * 16 + 255) // 256 * 256
    # F*C_in = 6: a multiple of 2 only
    assert fc.foldconv_plan(1, 32, 32, 3, 16, 3, 3, 1, 2, "float32").shapes.conv_kernel == 2
    # a 16-bit layer whose F*C_in is a multiple of 4 only: streaming kernel, 8-byte chunks of 4 rows
    s = fc.foldconv_plan(4, 60, 300, 3, 64, 3, 3, 1, 4, "float16").shapes
    assert s.conv_kernel == 2 and s.filter_compact_bytes == (4 * 3 * ((4 - 1 + 9 + 3) // 4) * 64 * 8 + 255) // 256 * 256
    assert s.workspace_bytes >= s.w_exp_bytes
    # ... but only where the output side still has whole 16-byte chunks (F*C_out a multiple of 8)
    assert fc.foldconv_plan(4, 60, 300, 3, 5, 3, 3, 1, 4, "float16").shapes.conv_kernel == 0
    # the gather kernel (channels off the chunk alignment) reads the original filter itself
    s = fc.foldconv_plan(1, 32, 32, 3, 16, 3, 3, 1, 1, "float32").shapes
    assert s.conv_kernel == 0 and s.filter_compact_bytes == (s.w_bytes + 255) // 256 * 256


def test_workloads_shapes():
    from paper_2601_11608_amd import workloads as wl

    assert [l.F for l in wl.CONFIGS["c5"]] == [16, 4, 4, 4, 4]
    layers, x, ws, bs = wl.make_config("c1")
    assert tuple(x.shape) == (1, 32, 32, 3) and tuple(ws[0].shape) == (3, 3, 3, 16) and bs[0] is None
    layers, x, ws, bs = wl.make_config("c4", N=2)
    assert tuple(x.shape) == (2, 1, 16000, 1) and tuple(ws[0].shape) == (1, 9, 1, 64)
    layers, x2, ws2, _ = wl.make_config("c4", N=2)
    assert (x2 == x).all() and (ws2[0] == ws[0]).all()      # seeded


def test_gemm_plan_is_a_folded_one_by_one_conv(fc):
    """paper: "Generalization to GEMM via 1x1 Convolution"."""
    p = fc.foldconv_plan_gemm(1 << 20, 12, 64, 4, "float16")
    s = p.shapes
    assert (s.KH, s.KW, s.pad_h, s.pad_w, s.KW_fold, s.d_min, s.d_max) == (1, 1, 0, 0, 1, 0, 0)
    assert s.N * s.H * s.W == 1 << 20 and s.W % 4 == 0 and s.C_in == 12 and s.C_out == 64
    assert (s.C_fold, s.Co_fold) == (48, 256) and s.unfold_is_alias == 1
    assert s.useful_flops == 2.0 * (1 << 20) * 12 * 64
    assert s.x_bytes == (1 << 20) * 12 * 2 and s.y_bytes == (1 << 20) * 64 * 2
    assert s.W_out_fold < 65000 and s.W_out < 65000   # rows short enough for the vector kernels, folded or not
    assert s.padded_kernel == 2            # so the zero-padded reference streams as well
    with pytest.raises(fc.FoldconvError) as e:
        fc.foldconv_plan_gemm(1001, 12, 64, 4, "float16")
    assert e.value.status == -2
    # a prime row count still plans (one long image row)
    s = fc.foldconv_plan_gemm(7919, 8, 16, 1, "float16").shapes
    assert s.H * s.W == 7919


def test_fold_factor_choice(fc):
    """Cost model: fold small misaligned C_in up to the chunk alignment, leave aligned wide layers alone."""
    # C_in = 3 or 1: no factor below 8 makes F*C_in a multiple of 8; a larger F only grows the filter
    assert fc.foldconv_choose_fold(64, 224, 224, 3, 64, 3, 3, 1, "float16") == 8
    assert fc.foldconv_choose_fold(16, 1, 16000, 1, 64, 1, 9, 4, "float16") == 8
    # C_in = 12: aligned from F = 2 on, but F*C_out = 96 fills only one and a half 64-column waves; F = 4 fills three
    assert fc.foldconv_choose_fold(32, 112, 112, 12, 48, 3, 3, 1, "bfloat16") == 4
    # a layer that is aligned and fills its tiles is left alone
    assert fc.foldconv_choose_fold(8, 56, 56, 64, 256, 3, 3, 1, "float16") == 1
    # width not divisible by 2: nothing to choose from
    assert fc.foldconv_choose_fold(1, 8, 9, 3, 4, 3, 3, 1, "float16") == 1
    for F in (8, 16):                      # every choice must be a legal plan
        fc.foldconv_plan(64, 224, 224, 3, 64, 3, 3, 1, F, "float16")
    lib = fc.load_library()
    assert lib.foldconv_choose_fold(1, 8, 8, 3, 4, 3, 3, 1, 1, None) == -1


def test_fold_factor_choice_against_the_measured_table(fc):
    """tests/golden/fold_choice_measured.json holds the times bench.py measured on an MI355X for every legal
    power-of-two fold factor of the benchmark layers.  The model's pick must be within 5 % of the fastest
    measured factor on every layer, and its estimate within 45 % of the measurement for every factor that
    runs a vector kernel (the model's constants were fitted to this table)."""
    import json

    table = json.load(open(os.path.join(ROOT, "tests", "golden", "fold_choice_measured.json")))["layers"]
    assert len(table) == 10                     # eight 16-bit layers, the small fp32 configuration, the headline shape in fp32
    for name, row in table.items():
        meas = {int(F): t for F, t in row["measured_us"].items() if t is not None}
        pick = fc.foldconv_choose_fold(*row["args"], row["dtype"])
        assert pick in meas, (name, pick)
        best = min(meas.values())
        assert meas[pick] <= 1.05 * best, (name, pick, meas)
        for F, t in meas.items():
            args = row["args"]
            s = fc.foldconv_plan(*args, F, row["dtype"]).shapes
            if s.conv_kernel != 0:
                assert abs(s.model_seconds * 1e6 - t) <= 0.45 * t, (name, F, s.model_seconds * 1e6, t)


def test_model_estimate_is_reported_per_plan(fc):
    """shapes.model_seconds is what foldconv_choose_fold compares: the pick has the smallest estimate."""
    args = (64, 224, 224, 3, 64, 3, 3, 1)
    pick = fc.foldconv_choose_fold(*args, "float16")
    est = {F: fc.foldconv_plan(*args, F, "float16").shapes.model_seconds for F in (1, 2, 4, 8, 16, 32)}
    assert all(v > 0 for v in est.values())
    assert est[pick] == min(est.values())


def _tiled_issued_flops(M, C, Co, F, KH, KW, pad, bn):
    """MFMA flops of the LDS-tiled kernel's band walk with `bn`-column tiles: for every tile the
    32-wide K blocks between the first and last extended channel its output slots can touch
    (rounded outwards to 8), plus the one 16-wide step of the rank-1 bias product, times the whole
    tile width (the plan's own accounting rule, restated here for the expected values below)."""
    FC, NCo = F * C, F * Co
    e_min, e_max = -((pad + F - 1) // F) * FC, ((F + KW - 2 - pad) // F + 1) * FC
    total = 0.0
    for n0 in range(0, NCo, bn):
        n1 = min(n0 + bn, NCo)
        g0, g1 = n0 // Co, (n1 - 1) // Co
        lo = max(e_min, ((g0 - pad) * C) // 8 * 8)
        hi = min(e_max, -(-((g1 + KW - pad) * C) // 8) * 8)
        blocks = -(-(hi - lo) // 32)
        total += 2.0 * M * bn * (blocks * 32 * KH + 16)
    return total


def test_tile_width_of_the_tiled_kernel_follows_the_issued_work(fc):
    """The 5-layer stack's MFMA-bound layers: 192-column tiles where they issue the least work
    (F*C_out = 144 in one tile; 528 = 3 x 192 with 8 % padding), 128 for 272 columns, 256 for 1024."""
    M = 32 * 112 * 28
    for C, Co, bn in ((20, 36, 192), (36, 68, 128), (68, 132, 192), (132, 256, 256)):
        s = fc.foldconv_plan(32, 112, 112, C, Co, 3, 3, 1, 4, "bfloat16").shapes
        assert s.conv_kernel == 1  # tiled
        want = _tiled_issued_flops(M, C, Co, 4, 3, 3, 1, bn)
        assert abs(s.issued_flops_band - want) <= 1e-9 * want, (C, Co, bn, s.issued_flops_band, want)
    # the two layers where the widths issue different amounts of work: the choice is the cheaper one by weight
    assert _tiled_issued_flops(M, 68, 132, 4, 3, 3, 1, 192) < _tiled_issued_flops(M, 68, 132, 4, 3, 3, 1, 128)
    assert _tiled_issued_flops(M, 36, 68, 4, 3, 3, 1, 128) < 0.93 * _tiled_issued_flops(M, 36, 68, 4, 3, 3, 1, 192)
