"""GPU parity: every step of the hot path, called through the C ABI, against
the fp64 CPU oracle on the same seeded inputs.  Data movement must be
bit-exact; convolution results must stay within the relative-L2 tolerances
(fp16 2e-3, bf16 8e-3, fp32 1e-5; maximum over images)."""
import numpy as np
import pytest
import torch

from helpers import (TOL, TORCH_DT, assert_elementwise, assert_same_to_rounding, bits, bits_as_f64, f64,
                     rel_l2_per_image)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fc():
    import paper_2601_11608_amd as fc

    fc.load_library()          # raises if the HIP library is not built: there is no fallback
    assert torch.cuda.is_available()
    return fc


def dev(t):
    return None if t is None else t.cuda()


def draw(shape, dt, seed, kind="normal"):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    t = torch.randn(shape, generator=g) if kind == "normal" else torch.rand(shape, generator=g) * 2 - 1
    return t.to(TORCH_DT[dt])


def abs_sum(oracle, x, w, b, ph, pw):
    """S = sum |x| |w| + |b| per output element (the oracle on absolute values): scale of the
    element-wise accumulation bound."""
    return oracle.conv_direct(np.abs(f64(x)), np.abs(f64(w)), None if b is None else np.abs(f64(b)), ph, pw, False)


def run_folded(fc, plan, x, w, b, flags=0, separate_fold=False):
    """expand -> fold -> forward through the ABI; returns y (CPU tensor)."""
    s = plan.shapes
    dt = x.dtype
    xd, wd, bd = dev(x), dev(w), dev(b)
    w_exp = torch.empty(s.w_exp_bytes // s.elem_bytes, dtype=dt, device="cuda")
    fc.foldconv_expand_filter(plan, wd, w_exp)
    if separate_fold:
        x_fold = torch.empty_like(xd)
        fc.foldconv_fold_input(plan, xd, x_fold)
    else:
        x_fold = xd
        fc.foldconv_fold_input(plan, xd, x_fold)        # alias: legal no-op
    ws = torch.empty(max(int(s.workspace_bytes), 256), dtype=torch.uint8, device="cuda")
    if flags & fc.FLAG_KEEP_FOLDED:
        y = torch.full((s.N, s.H_out, s.W_out_fold, s.Co_fold), float("nan"), dtype=dt, device="cuda")
    else:
        y = torch.full((s.N, s.H_out, s.W_out, s.C_out), float("nan"), dtype=dt, device="cuda")
    fc.foldconv_forward(plan, x_fold, w_exp, bd, y, ws, flags)
    torch.cuda.synchronize()
    return y.cpu()


def run_padded(fc, plan, x, w, b, flags=0):
    s = plan.shapes
    ws = torch.empty(max(int(s.padded_workspace_bytes), 256), dtype=torch.uint8, device="cuda")
    y = torch.full((s.N, s.H_out, s.W_out, s.C_out), float("nan"), dtype=x.dtype, device="cuda")
    fc.conv_padded_forward(plan, dev(x), dev(w), dev(b), y, ws, flags)
    torch.cuda.synchronize()
    return y.cpu()


# N, H, W, C, Co, KH, KW, pad, F, bias, relu  -- several tiles plus ragged tails in m and n
SMALL = [
    (2, 9, 24, 3, 5, 3, 3, 1, 8, True, False),      # FC=24, n ragged (40), m ragged (54)
    (1, 32, 32, 3, 16, 3, 3, 1, 8, False, False),   # the small fp32 benchmark layer
    (3, 7, 32, 3, 64, 3, 3, 1, 16, True, True),     # headline layer's structure, tiny
    (2, 12, 16, 12, 48, 3, 3, 1, 4, False, True),   # FC=48, NCo=192
    (2, 1, 256, 1, 64, 1, 9, 4, 32, False, False),  # Conv1d
    (1, 40, 64, 1, 1, 5, 1, 0, 8, True, False),     # the paper's K x 1 / VALID listing shape
    (1, 6, 12, 2, 3, 3, 3, 0, 4, True, False),      # VALID: ragged W_out (10)
    (1, 5, 12, 2, 2, 2, 4, 2, 4, False, False),     # even kernel, W_out = 13 > W
    (2, 5, 7, 3, 3, 3, 3, 1, 1, True, True),        # F = 1, unaligned channels
    (1, 9, 16, 20, 36, 3, 3, 1, 4, False, True),    # FC=80
    (1, 6, 8, 36, 68, 3, 3, 1, 4, False, False),    # FC=144, NCo=272
    (1, 3, 64, 1, 8, 1, 3, 1, 64, True, False),     # F == W
    (1, 4, 16, 5, 7, 1, 1, 0, 8, True, False),      # 1x1 (GEMM as conv), FC=40
    (1, 5, 8, 68, 132, 3, 3, 1, 4, True, True),     # FC=272, NCo=528: K too large for the streaming kernel
    (2, 3, 8, 132, 40, 3, 3, 1, 4, False, False),   # FC=528, NCo=160: ragged N tile of the tiled kernel
    (1, 20, 28, 68, 32, 3, 3, 1, 4, True, True),    # several 128-pixel M tiles, ragged last one
    (1, 6, 16, 68, 64, 3, 3, 1, 4, True, True),     # NCo = 256: the 256-column tile of the tiled kernel
    (1, 20, 28, 132, 256, 3, 3, 1, 4, False, True), # NCo = 1024, several M tiles with a ragged last one
    (1, 20, 28, 68, 132, 3, 3, 1, 4, True, True),   # NCo = 528: three 192-column tiles, the last one ragged, two M tiles
    (2, 10, 28, 20, 36, 3, 3, 1, 4, False, True),   # NCo = 144 in one 192-column tile
    (2, 65, 1024, 3, 64, 3, 3, 1, 16, True, True),  # 8320 folded pixels, many tiles per wave of the streaming kernel
    (3, 50, 480, 12, 48, 3, 3, 1, 4, False, False), # same with NCo = 192 (3 column groups)
    # 512 tiles or more: the streaming kernels deal them to the 8 XCDs in chunks
    (9, 131, 224, 3, 64, 3, 3, 1, 16, True, True),  # 516 tiles, the last ragged; chunks of 2 (14 pixels per row)
    (40, 1, 16000, 1, 64, 1, 9, 4, 32, False, False),  # Conv1d, 625 tiles, no rows to share
    (2, 40, 448, 8, 64, 3, 3, 1, 1, True, False),   # F = 1 on aligned channels: 14 tiles per row, chunks of 64
]


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("case", SMALL, ids=lambda c: "x".join(map(str, c[:9])))
def test_forward_small_matches_oracle(fc, oracle, case, dt):
    N, H, W, C, Co, KH, KW, pad, F, hb, relu = case
    x = draw((N, H, W, C), dt, 1)
    w = draw((KH, KW, C, Co), dt, 2) * (1.0 / np.sqrt(KH * KW * C))
    w = w.to(TORCH_DT[dt])
    b = draw((Co,), dt, 3) if hb else None
    ph, pw = oracle.axis_pads(KH, KW, pad)
    ref = oracle.conv_direct(f64(x), f64(w), None if b is None else f64(b), ph, pw, relu)
    S, K = abs_sum(oracle, x, w, b, ph, pw), KH * KW * C
    plan = fc.foldconv_plan(N, H, W, C, Co, KH, KW, pad, F, x.dtype)
    rflag = fc.FLAG_RELU if relu else 0
    y_band = run_folded(fc, plan, x, w, b, rflag)
    assert rel_l2_per_image(f64(y_band), ref) <= TOL[dt]
    assert_elementwise(f64(y_band), ref, S, K, dt, "band")
    y_dense = run_folded(fc, plan, x, w, b, rflag | fc.FLAG_DENSE_K, separate_fold=True)
    assert rel_l2_per_image(f64(y_dense), ref) <= TOL[dt]
    assert_elementwise(f64(y_dense), ref, S, K, dt, "dense")
    # skipping structural zeros only drops exact-zero products; what remains is summed in a
    # different fp32 order inside the MFMA (other K slots), so the two agree to the last rounding:
    # no element further apart than one output spacing, and only a few apart at all
    assert_same_to_rounding(f64(y_band), f64(y_dense), S, K, dt, "band vs dense")
    # folded layout + explicit reconstruct == fused reconstruct, bit for bit
    y_fold = run_folded(fc, plan, x, w, b, rflag | fc.FLAG_KEEP_FOLDED)
    s = plan.shapes
    y2 = torch.full((N, s.H_out, s.W_out, Co), float("nan"), dtype=x.dtype, device="cuda")
    fc.foldconv_unfold_output(plan, y_fold.cuda(), y2)
    torch.cuda.synchronize()
    assert np.array_equal(bits(y2), bits(y_band))
    want = oracle.unfold_output(bits_as_f64(y_fold), F, Co, s.W_out)
    assert np.array_equal(bits_as_f64(y2), want)
    # zero-padded reference path
    y_pad = run_padded(fc, plan, x, w, b, rflag)
    assert rel_l2_per_image(f64(y_pad), ref) <= TOL[dt]
    assert_elementwise(f64(y_pad), ref, S, K, dt, "padded")


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("KH,KW,C,Co,F,pad", [(3, 3, 3, 64, 16, 1), (1, 9, 1, 64, 32, 4), (5, 1, 1, 1, 8, 0),
                                               (3, 3, 12, 48, 4, 1), (2, 4, 2, 3, 4, 2), (3, 3, 3, 5, 1, 1),
                                               (3, 3, 132, 256, 4, 1)])
def test_expand_filter_bit_exact(fc, oracle, KH, KW, C, Co, F, pad, dt):
    w = draw((KH, KW, C, Co), dt, 11)
    plan = fc.foldconv_plan(1, 8, 8 * F, C, Co, KH, KW, pad, F, w.dtype)
    s = plan.shapes
    w_exp = torch.full((KH, s.KW_fold, F * C, F * Co), float("nan"), dtype=w.dtype, device="cuda")
    fc.foldconv_expand_filter(plan, w.cuda(), w_exp)
    torch.cuda.synchronize()
    want = oracle.expand_filter(bits_as_f64(w), F, s.pad_w)     # zeros are bit pattern 0 == +0.0
    assert np.array_equal(bits_as_f64(w_exp), want)


def run_compact(fc, plan, x, w, b, flags=0):
    """compact filter straight from w (no expanded filter anywhere) -> forward; returns y (CPU tensor)."""
    s = plan.shapes
    ws = torch.full((max(int(s.filter_compact_bytes), 256),), 0xFF, dtype=torch.uint8, device="cuda")
    fc.foldconv_pack_filter_compact(plan, dev(w), ws)
    if flags & fc.FLAG_KEEP_FOLDED:
        y = torch.full((s.N, s.H_out, s.W_out_fold, s.Co_fold), float("nan"), dtype=x.dtype, device="cuda")
    else:
        y = torch.full((s.N, s.H_out, s.W_out, s.C_out), float("nan"), dtype=x.dtype, device="cuda")
    fc.foldconv_forward(plan, dev(x), None, dev(b), y, ws, flags | fc.FLAG_FILTER_COMPACT)
    torch.cuda.synchronize()
    return y.cpu()


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("case", SMALL, ids=lambda c: "x".join(map(str, c[:9])))
def test_forward_compact_filter(fc, oracle, case, dt):
    """Only the non-zero blocks of w' are stored; the same values reach the same MFMA slots, so
    the result equals the packed-w' route bit for bit, and the oracle within tolerance."""
    N, H, W, C, Co, KH, KW, pad, F, hb, relu = case
    x = draw((N, H, W, C), dt, 1)
    w = (draw((KH, KW, C, Co), dt, 2) * (1.0 / np.sqrt(KH * KW * C))).to(TORCH_DT[dt])
    b = draw((Co,), dt, 3) if hb else None
    ph, pw = oracle.axis_pads(KH, KW, pad)
    ref = oracle.conv_direct(f64(x), f64(w), None if b is None else f64(b), ph, pw, relu)
    plan = fc.foldconv_plan(N, H, W, C, Co, KH, KW, pad, F, x.dtype)
    rflag = fc.FLAG_RELU if relu else 0
    for extra in (0, fc.FLAG_DENSE_K, fc.FLAG_KEEP_FOLDED):
        y_c = run_compact(fc, plan, x, w, b, rflag | extra)
        y_p = run_folded(fc, plan, x, w, b, rflag | extra)
        if dt == "f32" and extra == fc.FLAG_DENSE_K and not np.array_equal(bits(y_c), bits(y_p)):
            # fp32 has no tiled kernel: a dense walk of the packed filter too long for the streaming
            # instances runs the element-gather kernel, while the compact form walks the band on the
            # streaming kernel: another summation order, the same result within the rounding bound
            assert_elementwise(f64(y_c), ref, abs_sum(oracle, x, w, b, ph, pw), KH * KW * C, dt, "compact dense")
            assert_elementwise(f64(y_p), ref, abs_sum(oracle, x, w, b, ph, pw), KH * KW * C, dt, "packed dense")
            continue
        assert np.array_equal(bits(y_c), bits(y_p)), extra
        if not extra:
            assert rel_l2_per_image(f64(y_c), ref) <= TOL[dt]
            assert_elementwise(f64(y_c), ref, abs_sum(oracle, x, w, b, ph, pw), KH * KW * C, dt, "compact")


# Dense walks served by the LDS-staged streaming kernel (KH = 3, F*C_in = 48 with KW' = 3, F*C_out a
# multiple of 256): N, H, W, C, Co, F, bias, relu
DENSE_LDS = [
    (1, 5, 48, 3, 16, 16, True, False),      # 15 folded pixels: one ragged tile, one 256-column group
    (2, 33, 96, 3, 32, 16, False, True),     # 396 pixels: 13 tiles, the last ragged; two column groups
    (1, 64, 1024, 3, 64, 16, True, True),    # 4096 pixels = 128 tiles: several per workgroup, four column groups
    (3, 20, 160, 6, 64, 8, True, False),     # F = 8, C_in = 6
    (2, 17, 64, 12, 64, 4, False, False),    # F = 4, C_in = 12: F*C_out = 256
    (40, 9, 32, 3, 128, 16, True, True),     # 8 column groups, tiles spanning images
]


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("case", DENSE_LDS, ids=lambda c: "x".join(map(str, c[:6])))
def test_dense_walk_with_staged_input(fc, oracle, case, dt):
    """FLAG_DENSE_K on shapes whose whole K extent is register-resident: every K-step of w' is
    multiplied (structural zeros included), input tiles shared through LDS.  Checked against the
    oracle, against the band walk, with the compact filter (bit-identical) and kept folded."""
    N, H, W, C, Co, F, hb, relu = case
    x = draw((N, H, W, C), dt, 61)
    w = (draw((3, 3, C, Co), dt, 62) * (1.0 / np.sqrt(9 * C))).to(TORCH_DT[dt])
    b = draw((Co,), dt, 63) if hb else None
    ref = oracle.conv_direct(f64(x), f64(w), None if b is None else f64(b), 1, 1, relu)
    plan = fc.foldconv_plan(N, H, W, C, Co, 3, 3, 1, F, x.dtype)
    s = plan.shapes
    assert s.conv_kernel == 2 and s.C_fold == 48 and s.KW_fold == 3 and s.Co_fold % 256 == 0
    print("dense staged", case, dt, flush=True)
    rflag = fc.FLAG_RELU if relu else 0
    y_dense = run_folded(fc, plan, x, w, b, rflag | fc.FLAG_DENSE_K)
    assert not bool(torch.isnan(y_dense).any()), "unwritten output elements"
    assert rel_l2_per_image(f64(y_dense), ref) <= TOL[dt]
    S, K = abs_sum(oracle, x, w, b, 1, 1), 9 * C
    assert_elementwise(f64(y_dense), ref, S, K, dt, "dense (staged input)")
    y_band = run_folded(fc, plan, x, w, b, rflag)
    assert_same_to_rounding(f64(y_band), f64(y_dense), S, K, dt, "band vs dense (staged input)")
    y_c = run_compact(fc, plan, x, w, b, rflag | fc.FLAG_DENSE_K)
    assert np.array_equal(bits(y_c), bits(y_dense))
    y_f = run_folded(fc, plan, x, w, b, rflag | fc.FLAG_DENSE_K | fc.FLAG_KEEP_FOLDED)
    assert np.array_equal(bits(y_f).reshape(-1), bits(y_dense).reshape(-1))       # the reconstruct is an alias here


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("KH,KW,C,Co,F,pad", [(3, 3, 3, 64, 16, 1), (1, 9, 1, 64, 32, 4), (5, 1, 1, 1, 8, 0),
                                               (3, 3, 12, 48, 4, 1), (2, 4, 2, 8, 4, 2), (3, 3, 132, 256, 4, 1),
                                               (3, 3, 20, 36, 4, 1), (1, 1, 5, 7, 8, 0), (3, 5, 6, 10, 4, 2),
                                               # F*C_in = 12, 12, 4: chunks of 4 rows (8 bytes)
                                               (3, 3, 3, 64, 4, 1), (3, 3, 6, 24, 2, 1), (1, 7, 2, 40, 2, 3)])
def test_compact_filter_holds_the_band_of_the_expanded_filter(fc, oracle, KH, KW, C, Co, F, pad, dt):
    """Every chunk (8 rows, or 4 where F*C_in is a multiple of 4 only) of every column of the oracle's
    expanded filter is either all zero or found, bit for bit, where the compact layout says it is;
    the compact form is much smaller."""
    w = draw((KH, KW, C, Co), dt, 12)
    plan = fc.foldconv_plan(1, 8, 8 * F, C, Co, KH, KW, pad, F, w.dtype)
    s = plan.shapes
    assert s.conv_kernel != 0                    # a vector kernel: chunked compact storage
    ws = torch.full((int(s.filter_compact_bytes),), 0xFF, dtype=torch.uint8, device="cuda")
    fc.foldconv_pack_filter_compact(plan, w.cuda(), ws)
    torch.cuda.synchronize()
    E = 8 if (F * C) % 8 == 0 else 4
    g8 = int(np.gcd(C, E))
    P, cJ = E // g8, (E - g8 + KW * C + E - 1) // E
    assert s.filter_compact_bytes == -(-P * KH * cJ * Co * 2 * E // 256) * 256
    cpk = ws.cpu().numpy().view(np.int16)[: P * KH * cJ * Co * E].reshape(P, KH, cJ, Co, E)
    w_exp = oracle.expand_filter(bits_as_f64(w), F, s.pad_w).astype(np.int16)        # [KH, KW', FC, FCo] bit patterns
    w_exp = w_exp.reshape(KH, s.KW_fold * F * C, F * Co)
    e_min = s.d_min * F * C
    used = np.zeros((P, KH, cJ, Co), dtype=bool)
    for g in range(F):
        a = (g - s.pad_w) * C - e_min
        assert a >= 0
        for q in range(w_exp.shape[1] // E):
            rows = w_exp[:, E * q:E * q + E, g * Co:(g + 1) * Co]                      # [KH, E, Co]
            j = q - a // E
            if 0 <= j < cJ:
                assert np.array_equal(cpk[(a % E) // g8, :, j].transpose(0, 2, 1), rows), (g, q)
                used[(a % E) // g8, :, j] = True
            else:
                assert not rows.any(), (g, q)
    if F >= P:                                   # every phase copy serves some slot: what no slot reads is padding
        assert not cpk[~used].any()
    if s.w_exp_bytes >= 4096:                    # beyond the 16-byte chunk and 256-byte rounding effects
        assert s.filter_compact_bytes < s.w_exp_bytes


@pytest.mark.parametrize("dt", ["f16", "f32"])
@pytest.mark.parametrize("N,H,W,C,F", [(2, 5, 48, 3, 16), (1, 1, 16000, 1, 32), (3, 7, 20, 5, 4), (1, 3, 6, 1, 2)])
def test_fold_input_bit_exact(fc, oracle, N, H, W, C, F, dt):
    x = draw((N, H, W, C), dt, 12)
    plan = fc.foldconv_plan(N, H, W, C, 4, 1, 1, 0, F, x.dtype)
    xf = torch.full((N, H, W // F, F * C), float("nan"), dtype=x.dtype, device="cuda")
    fc.foldconv_fold_input(plan, x.cuda(), xf)
    torch.cuda.synchronize()
    assert np.array_equal(bits_as_f64(xf), oracle.fold_input(bits_as_f64(x), F))


def test_fold_input_unaligned_pointers(fc, oracle):
    """Odd byte offsets take the byte-wise copy."""
    x = draw((1, 3, 8, 3), "f16", 13)
    plan = fc.foldconv_plan(1, 3, 8, 3, 4, 1, 1, 0, 4, x.dtype)
    buf_in = torch.zeros(x.numel() + 8, dtype=x.dtype, device="cuda")
    buf_out = torch.zeros(x.numel() + 8, dtype=x.dtype, device="cuda")
    buf_in[1:1 + x.numel()] = x.cuda().flatten()
    fc.foldconv_fold_input(plan, buf_in.data_ptr() + 2, buf_out.data_ptr() + 6)
    torch.cuda.synchronize()
    got = buf_out[3:3 + x.numel()].reshape(1, 3, 2, 12)
    assert np.array_equal(bits_as_f64(got), oracle.fold_input(bits_as_f64(x), 4))
    assert float(buf_out[:3].abs().sum()) == 0 and float(buf_out[3 + x.numel():].abs().sum()) == 0


def test_runtime_argument_errors(fc):
    plan = fc.foldconv_plan(1, 6, 12, 2, 3, 3, 3, 0, 4, torch.float16)     # ragged: unfold is not an alias
    s = plan.shapes
    assert s.unfold_is_alias == 0
    yf = torch.zeros(s.y_fold_bytes // 2, dtype=torch.float16, device="cuda")
    with pytest.raises(fc.FoldconvError) as e:
        fc.foldconv_unfold_output(plan, yf, yf)
    assert e.value.status == -1
    with pytest.raises(fc.FoldconvError) as e:
        fc.conv_padded_forward(plan, yf, yf, None, yf, torch.zeros(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -4


def test_empty_bias_and_relu_flags(fc, oracle):
    """b = const, w = 0 -> y == b (paper: Eq. bias_construct); ReLU clamps."""
    N, H, W, C, Co, F = 1, 4, 16, 3, 4, 8
    x = draw((N, H, W, C), "f16", 14)
    w = torch.zeros((3, 3, C, Co), dtype=torch.float16)
    b = torch.tensor([0.5, -1.25, 2.0, -0.0], dtype=torch.float16)
    plan = fc.foldconv_plan(N, H, W, C, Co, 3, 3, 1, F, x.dtype)
    y = run_folded(fc, plan, x, w, b, 0)
    assert torch.equal(y, b.expand(N, H, W, Co))
    y = run_folded(fc, plan, x, w, b, fc.FLAG_RELU)
    assert torch.equal(y, torch.relu(b).expand(N, H, W, Co))


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("M,K,N,F", [(4096, 12, 64, 4), (1000, 3, 40, 8), (8192 * 3, 5, 16, 8), (777, 24, 8, 1)])
def test_gemm_as_folded_one_by_one_conv(fc, oracle, M, K, N, F, dt):
    """paper: "Generalization to GEMM via 1x1 Convolution": C = A B with tall-skinny A."""
    A = draw((M, K), dt, 21)
    B = (draw((K, N), dt, 22) * (1.0 / np.sqrt(K))).to(TORCH_DT[dt])
    plan = fc.foldconv_plan_gemm(M, K, N, F, A.dtype)
    s = plan.shapes
    x = A.reshape(1, s.H, s.W, K)
    w = B.reshape(1, 1, K, N)
    ref = oracle.conv_direct(f64(x), f64(w), None, 0, 0).reshape(1, M, N)     # pinned to A @ B in the oracle tests
    S = abs_sum(oracle, x, w, None, 0, 0).reshape(1, M, N)
    y = run_folded(fc, plan, x, w, None, 0).reshape(1, M, N)
    assert rel_l2_per_image(f64(y), ref) <= TOL[dt]
    assert_elementwise(f64(y), ref, S, K, dt, "gemm folded")
    yp = run_padded(fc, plan, x, w, None, 0).reshape(1, M, N)
    assert rel_l2_per_image(f64(yp), ref) <= TOL[dt]
    assert_elementwise(f64(yp), ref, S, K, dt, "gemm padded")


def _random_cases(n, seed):
    """Seeded random geometries: small enough for the oracle, varied enough to reach all three kernels,
    ragged tiles in m and n, VALID / 'same' / over-padded, even and odd kernels, F from 1 to W."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        F = int(rng.choice([1, 2, 4, 8, 16]))
        Wf = int(rng.integers(1, 9))
        W = F * Wf
        H = int(rng.integers(1, 12))
        C = int(rng.choice([1, 2, 3, 4, 6, 8, 12, 20, 36, 66]))
        Co = int(rng.choice([1, 3, 8, 16, 20, 40, 64, 72]))
        KH = int(rng.integers(1, min(H, 5) + 1))
        KW = int(rng.integers(1, 6))
        pad = int(rng.integers(0, 3))
        N = int(rng.integers(1, 4))
        ph, pw = (pad if KH > 1 else 0), (pad if KW > 1 else 0)
        if H + 2 * ph - KH + 1 <= 0 or W + 2 * pw - KW + 1 <= 0:
            continue
        if N * H * W * Co * KH * KW * C > 3e8:
            continue
        out.append((N, H, W, C, Co, KH, KW, pad, F, bool(rng.integers(0, 2)), bool(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("chunk", range(6))
def test_random_geometries(fc, oracle, chunk, dt):
    kernels = set()
    for case in _random_cases(25, 1000 + chunk):
        N, H, W, C, Co, KH, KW, pad, F, hb, relu = case
        x = draw((N, H, W, C), dt, 41)
        w = (draw((KH, KW, C, Co), dt, 42) * (1.0 / np.sqrt(KH * KW * C))).to(TORCH_DT[dt])
        b = draw((Co,), dt, 43) if hb else None
        ph, pw = oracle.axis_pads(KH, KW, pad)
        ref = oracle.conv_direct(f64(x), f64(w), None if b is None else f64(b), ph, pw, relu)
        plan = fc.foldconv_plan(N, H, W, C, Co, KH, KW, pad, F, x.dtype)
        kernels.add(plan.shapes.conv_kernel)
        rflag = fc.FLAG_RELU if relu else 0
        S, K = abs_sum(oracle, x, w, b, ph, pw), KH * KW * C
        for name, y in (("band", run_folded(fc, plan, x, w, b, rflag)),
                        ("dense", run_folded(fc, plan, x, w, b, rflag | fc.FLAG_DENSE_K)),
                        ("compact", run_compact(fc, plan, x, w, b, rflag)),
                        ("padded", run_padded(fc, plan, x, w, b, rflag))):
            assert not bool(torch.isnan(y).any()), (case, name)
            # per-image relative L2 (an image that ReLU leaves all zero must come out all zero) and
            # the element-wise bound
            err = rel_l2_per_image(f64(y), ref)
            assert err <= TOL[dt], (case, name, err)
            assert_elementwise(f64(y), ref, S, K, dt, "%s %s" % (case, name))
    assert len(kernels) >= 2


@pytest.mark.parametrize("case", [(4, 64, 224, 3, 64, 3, 3, 1, 16, True, False),     # the headline layer's shape, 4 images
                                  (16, 64, 224, 3, 64, 3, 3, 1, 16, True, True),      # 16 images: bound by its MFMAs, 8-byte chunks
                                  (2, 40, 48, 12, 48, 3, 3, 1, 4, False, True),       # c3-like: several K-steps per kh
                                  (3, 1, 4000, 1, 64, 1, 9, 4, 32, True, False),      # 1-D, one input channel
                                  (1, 30, 64, 6, 10, 3, 3, 1, 2, True, True),         # F*C_out = 20: cropped columns
                                  (2, 24, 30, 3, 16, 3, 3, 1, 2, True, False),        # F*C_in = 6: 8-byte chunks only
                                  (2, 20, 24, 16, 32, 3, 3, 1, 1, False, True)],      # unfolded, C_in = 16: 16-byte chunks
                         ids=lambda c: "x".join(map(str, c[:9])))
def test_fp32_layers_on_the_streaming_kernel(fc, oracle, case):
    """fp32 tensors whose folded pixels are whole 8- or 16-byte chunks (F*C_in a multiple of 2 or 4)
    run the streaming kernel: steps of 4 or 8 K values as two or four MFMAs of K = 2, whichever walks
    fewer structural zeros, fp32 all the way (paper, appendix listing: the fp32 setting of its
    equivalence check).  Every walk and the zero-padded reference against the oracle, rel-L2 and
    element by element."""
    N, H, W, C, Co, KH, KW, pad, F, hb, relu = case
    dt = "f32"
    x = draw((N, H, W, C), dt, 71)
    w = (draw((KH, KW, C, Co), dt, 72) * (1.0 / np.sqrt(KH * KW * C))).to(TORCH_DT[dt])
    b = draw((Co,), dt, 73) if hb else None
    ph, pw = oracle.axis_pads(KH, KW, pad)
    ref = oracle.conv_direct(f64(x), f64(w), None if b is None else f64(b), ph, pw, relu)
    plan = fc.foldconv_plan(N, H, W, C, Co, KH, KW, pad, F, x.dtype)
    assert plan.shapes.conv_kernel == 2 and plan.shapes.workspace_bytes >= plan.shapes.w_exp_bytes
    rflag = fc.FLAG_RELU if relu else 0
    S, K = abs_sum(oracle, x, w, b, ph, pw), KH * KW * C
    y_band = run_folded(fc, plan, x, w, b, rflag)
    for name, y in (("band", y_band),
                    ("dense", run_folded(fc, plan, x, w, b, rflag | fc.FLAG_DENSE_K)),
                    ("compact", run_compact(fc, plan, x, w, b, rflag)),
                    ("padded", run_padded(fc, plan, x, w, b, rflag))):
        assert not bool(torch.isnan(y).any()), (case, name)
        err = rel_l2_per_image(f64(y), ref)
        print("fp32 %s %s: rel-L2 %.2e" % (case[:9], name, err), flush=True)
        assert err <= TOL[dt], (case, name, err)
        assert_elementwise(f64(y), ref, S, K, dt, "%s %s" % (case, name))
    # the compact filter feeds the same values to the same MFMA slots as the packed one
    assert np.array_equal(bits(run_compact(fc, plan, x, w, b, rflag)), bits(y_band))


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("case", [(4, 60, 300, 3, 64, 3, 3, 1, 4, True, False),      # W = 300 = 4 * 75: no fold reaches 8 channels
                                  (3, 28, 28, 1, 32, 3, 3, 1, 4, True, True),        # one input channel, W = 28 = 4 * 7
                                  (2, 33, 36, 6, 24, 3, 3, 1, 2, False, False),      # F*C_in = 12, several K-steps per kh
                                  (2, 20, 24, 20, 16, 3, 3, 1, 1, True, False),      # unfolded, C_in = 20: eight K-steps per kh
                                  (1, 1, 6000, 2, 40, 1, 7, 3, 2, False, True)],     # 1-D
                         ids=lambda c: "x".join(map(str, c[:9])))
def test_sixteen_bit_layers_in_eight_byte_chunks(fc, oracle, case, dt):
    """16-bit tensors whose folded channel count is a multiple of 4 but not of 8 run the streaming
    kernel with 8-byte operand chunks (K-steps of 8 on the 32x32x8 MFMA) instead of the element-gather
    kernel.  Every walk and the zero-padded reference against the oracle, rel-L2 and element by
    element (paper: Eq. new_conv_H; the alignment remark on F in the IR formulation)."""
    N, H, W, C, Co, KH, KW, pad, F, hb, relu = case
    assert (F * C) % 8 == 4
    x = draw((N, H, W, C), dt, 81)
    w = (draw((KH, KW, C, Co), dt, 82) * (1.0 / np.sqrt(KH * KW * C))).to(TORCH_DT[dt])
    b = draw((Co,), dt, 83) if hb else None
    ph, pw = oracle.axis_pads(KH, KW, pad)
    ref = oracle.conv_direct(f64(x), f64(w), None if b is None else f64(b), ph, pw, relu)
    plan = fc.foldconv_plan(N, H, W, C, Co, KH, KW, pad, F, x.dtype)
    assert plan.shapes.conv_kernel == 2 and plan.shapes.workspace_bytes >= plan.shapes.w_exp_bytes
    rflag = fc.FLAG_RELU if relu else 0
    S, K = abs_sum(oracle, x, w, b, ph, pw), KH * KW * C
    y_band = run_folded(fc, plan, x, w, b, rflag)
    y_compact = run_compact(fc, plan, x, w, b, rflag)
    for name, y in (("band", y_band),
                    ("dense", run_folded(fc, plan, x, w, b, rflag | fc.FLAG_DENSE_K)),
                    ("compact", y_compact),
                    ("compact dense", run_compact(fc, plan, x, w, b, rflag | fc.FLAG_DENSE_K)),
                    ("padded", run_padded(fc, plan, x, w, b, rflag))):
        assert not bool(torch.isnan(y).any()), (case, name)
        err = rel_l2_per_image(f64(y), ref)
        print("%s %s %s: rel-L2 %.2e" % (dt, case[:9], name, err), flush=True)
        assert err <= TOL[dt], (case, name, err)
        assert_elementwise(f64(y), ref, S, K, dt, "%s %s" % (case, name))
    # the compact filter feeds the same values to the same MFMA slots as the packed one
    assert np.array_equal(bits(y_compact), bits(y_band))


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("N,H,W,C,Co,KH,KW,pad", [(2, 9, 12, 8, 16, 3, 3, 1), (1, 6, 40, 16, 64, 1, 5, 2), (1, 7, 7, 64, 40, 3, 3, 0)])
def test_fold_factor_one_is_the_direct_path(fc, oracle, N, H, W, C, Co, KH, KW, pad, dt):
    """F = 1: the fold is the identity, the expanded filter is the filter itself, and with C_in
    already aligned the zero-padded reference pads nothing: both entry points must then produce the
    same bits (same kernel, same operands)."""
    x = draw((N, H, W, C), dt, 51)
    w = (draw((KH, KW, C, Co), dt, 52) * (1.0 / np.sqrt(KH * KW * C))).to(TORCH_DT[dt])
    b = draw((Co,), dt, 53)
    plan = fc.foldconv_plan(N, H, W, C, Co, KH, KW, pad, 1, x.dtype)
    s = plan.shapes
    assert (s.W_fold, s.C_fold, s.KW_fold, s.C_pad, s.C_out_pad) == (W, C, KW, C, Co)
    w_exp = torch.empty(s.w_exp_bytes // s.elem_bytes, dtype=x.dtype, device="cuda")
    fc.foldconv_expand_filter(plan, w.cuda(), w_exp)
    torch.cuda.synchronize()
    assert np.array_equal(bits(w_exp).reshape(-1), bits(w).reshape(-1))
    y_f = run_folded(fc, plan, x, w, b, fc.FLAG_RELU)
    y_p = run_padded(fc, plan, x, w, b, fc.FLAG_RELU)
    assert np.array_equal(bits(y_f), bits(y_p))
    ph, pw = oracle.axis_pads(KH, KW, pad)
    ref = oracle.conv_direct(f64(x), f64(w), f64(b), ph, pw, True)
    assert rel_l2_per_image(f64(y_f), ref) <= TOL[dt]
    assert_elementwise(f64(y_f), ref, abs_sum(oracle, x, w, b, ph, pw), KH * KW * C, dt, "F = 1")
