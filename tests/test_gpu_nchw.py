"""GPU parity of the channels-first front end (height or width folding of NCHW
tensors), through the C ABI, against the fp64 oracle's NCHW routines: the
three data-movement steps bit for bit, the whole path within the relative-L2
tolerances."""
import numpy as np
import pytest
import torch

from helpers import TOL, TORCH_DT, bits, bits_as_f64, f64, rel_l2_per_image

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fc():
    import paper_2601_11608_amd as fc

    fc.load_library()
    assert torch.cuda.is_available()
    return fc


def draw(shape, dt, seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return torch.randn(shape, generator=g).to(TORCH_DT[dt])


AXES = ["W", "H"]


def axis_code(fc, axis):
    return fc.FOLD_H if axis == "H" else fc.FOLD_W


# N, C, H, W, F (F divides the folded axis in both orientations)
FOLD_CASES = [(2, 3, 16, 32, 8), (1, 1, 64, 32, 32), (3, 5, 8, 12, 4), (1, 2, 6, 6, 2), (2, 12, 28, 20, 4), (1, 7, 5, 5, 1),
              # the LDS-tiled pass: a ragged last tile on either axis; rows so long that the tile height shrinks
              (2, 3, 40, 72, 8), (1, 12, 24, 224, 4)]


@pytest.mark.parametrize("dt", ["f16", "f32"])
@pytest.mark.parametrize("axis", AXES)
@pytest.mark.parametrize("N,C,H,W,F", FOLD_CASES)
def test_fold_input_nchw_bit_exact(fc, oracle, N, C, H, W, F, axis, dt):
    x = draw((N, C, H, W), dt, 21)
    plan = fc.foldconv_plan_nchw(N, C, H, W, 8, 3, 3, 1, F, axis_code(fc, axis), x.dtype)
    xf = torch.full((x.numel(),), float("nan"), dtype=x.dtype, device="cuda")
    fc.foldconv_fold_input_nchw(plan, x.cuda(), xf)
    torch.cuda.synchronize()
    xb = bits_as_f64(x)
    if axis == "H":
        want = oracle.fold_input_h_nchw(xb, F).transpose(0, 3, 2, 1)      # [N, W, H/F, F*C]
    else:
        want = oracle.fold_input(xb.transpose(0, 2, 3, 1), F)             # [N, H, W/F, F*C]
    assert np.array_equal(bits_as_f64(xf).reshape(want.shape), want)


@pytest.mark.parametrize("dt", ["bf16", "f32"])
@pytest.mark.parametrize("axis", AXES)
@pytest.mark.parametrize("Co,C,KH,KW,F,pad", [(64, 3, 3, 3, 16, 1), (8, 1, 9, 1, 32, 4), (5, 3, 3, 5, 4, 2), (3, 2, 4, 2, 4, 2),
                                               (48, 12, 3, 3, 4, 1), (7, 5, 1, 1, 8, 0)])
def test_expand_filter_oihw_bit_exact(fc, oracle, Co, C, KH, KW, F, pad, axis, dt):
    w = draw((Co, C, KH, KW), dt, 22)
    plan = fc.foldconv_plan_nchw(1, C, 8 * F, 8 * F, Co, KH, KW, pad, F, axis_code(fc, axis), w.dtype)
    s = plan.shapes
    w_exp = torch.full((s.w_exp_bytes // s.elem_bytes,), float("nan"), dtype=w.dtype, device="cuda")
    fc.foldconv_expand_filter_oihw(plan, w.cuda(), w_exp)
    torch.cuda.synchronize()
    wb = bits_as_f64(w)
    if axis == "H":
        p = pad if KH > 1 else 0
        want = oracle.expand_filter_h_oihw(wb, F, p).transpose(3, 2, 1, 0)   # [KW, KH', F*C, F*Co]
    else:
        p = pad if KW > 1 else 0
        want = oracle.expand_filter(wb.transpose(2, 3, 1, 0), F, p)          # [KH, KW', F*C, F*Co]
    assert s.pad_w == p
    assert np.array_equal(bits_as_f64(w_exp).reshape(want.shape), want)


# N, Co, H, W, KH, KW, pad, F: output extents ragged or not, tile path (Co % 8 == 0, output width % 8 == 0) or element path
UNFOLD_CASES = [(2, 64, 16, 64, 3, 3, 1, 16), (1, 128, 8, 72, 3, 3, 1, 8), (2, 8, 12, 16, 3, 3, 0, 4), (1, 5, 12, 12, 3, 3, 1, 4),
                (1, 16, 10, 20, 2, 4, 2, 5), (3, 72, 9, 9, 3, 3, 1, 3), (1, 64, 200, 8, 1, 1, 0, 8)]


@pytest.mark.parametrize("dt", ["f16", "f32"])
@pytest.mark.parametrize("axis", AXES)
@pytest.mark.parametrize("N,Co,H,W,KH,KW,pad,F", UNFOLD_CASES)
def test_unfold_output_nchw_bit_exact(fc, oracle, N, Co, H, W, KH, KW, pad, F, axis, dt):
    if (W if axis == "W" else H) % F:
        pytest.skip("fold factor does not divide this axis")
    plan = fc.foldconv_plan_nchw(N, 2, H, W, Co, KH, KW, pad, F, axis_code(fc, axis), TORCH_DT[dt])
    s = plan.shapes
    yf = draw((N, s.H_out, s.W_out_fold, F * Co), dt, 23)                   # plan-space folded output
    y = torch.full((N * Co * s.H_out * s.W_out,), float("nan"), dtype=yf.dtype, device="cuda")
    fc.foldconv_unfold_output_nchw(plan, yf.cuda(), y)
    torch.cuda.synchronize()
    yb = bits_as_f64(yf)
    if axis == "H":
        # plan rows are image columns: y'[n, w, h', g*Co+co] -> yh[n, g*Co+co, h', w]
        want = oracle.unfold_output_h_nchw(yb.transpose(0, 3, 2, 1), F, Co, s.W_out)     # [N, Co, H_out_img, W_out_img]
    else:
        want = oracle.unfold_output(yb, F, Co, s.W_out).transpose(0, 3, 1, 2)
    assert np.array_equal(bits_as_f64(y).reshape(want.shape), want)


def run_nchw(fc, plan, x, w, b, relu):
    s = plan.shapes
    dt = x.dtype
    w_exp = torch.empty(s.w_exp_bytes // s.elem_bytes, dtype=dt, device="cuda")
    fc.foldconv_expand_filter_oihw(plan, w.cuda(), w_exp)
    xf = torch.empty(x.numel(), dtype=dt, device="cuda")
    fc.foldconv_fold_input_nchw(plan, x.cuda(), xf)
    ws = torch.empty(max(int(s.workspace_bytes), 256), dtype=torch.uint8, device="cuda")
    yf = torch.full((s.y_fold_bytes // s.elem_bytes,), float("nan"), dtype=dt, device="cuda")
    fc.foldconv_forward(plan, xf, w_exp, None if b is None else b.cuda(), yf, ws,
                        fc.FLAG_KEEP_FOLDED | (fc.FLAG_RELU if relu else 0))
    y = torch.full((s.y_bytes // s.elem_bytes,), float("nan"), dtype=dt, device="cuda")
    fc.foldconv_unfold_output_nchw(plan, yf, y)
    torch.cuda.synchronize()
    return y.cpu()


# N, C, H, W, Co, KH, KW, pad, F, bias, relu
PIPE = [
    (2, 3, 32, 48, 64, 3, 3, 1, 16, True, True),     # headline structure
    (1, 1, 64, 64, 8, 5, 1, 0, 8, True, False),      # K x 1 VALID (the paper's proof setting when H is folded)
    (2, 12, 16, 24, 48, 3, 3, 1, 4, False, True),
    (1, 2, 12, 12, 3, 3, 3, 0, 4, True, False),      # VALID: ragged folded output, element path
    (1, 3, 16, 16, 16, 2, 4, 2, 4, False, False),    # even kernels: outputs larger than inputs
    (1, 68, 8, 8, 32, 3, 3, 1, 4, True, True),       # large K: tiled kernel
]


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("axis", AXES)
@pytest.mark.parametrize("case", PIPE, ids=lambda c: "x".join(map(str, c[:9])))
def test_nchw_path_matches_oracle(fc, oracle, case, axis, dt):
    N, C, H, W, Co, KH, KW, pad, F, hb, relu = case
    x = draw((N, C, H, W), dt, 31)
    w = (draw((Co, C, KH, KW), dt, 32) * (1.0 / np.sqrt(KH * KW * C))).to(TORCH_DT[dt])
    b = draw((Co,), dt, 33) if hb else None
    ph, pw = oracle.axis_pads(KH, KW, pad)
    ref = oracle.conv_direct_nchw(f64(x), f64(w), None if b is None else f64(b), ph, pw, relu)
    plan = fc.foldconv_plan_nchw(N, C, H, W, Co, KH, KW, pad, F, axis_code(fc, axis), x.dtype)
    assert plan.shapes.fold_axis == axis_code(fc, axis)
    y = run_nchw(fc, plan, x, w, b, relu).reshape(ref.shape)
    assert not bool(torch.isnan(y).any())
    assert rel_l2_per_image(f64(y), ref) <= TOL[dt]


@pytest.mark.parametrize("axis", AXES)
def test_nchw_headline_layer_full_size(fc, oracle, axis):
    """The headline layer handed over channels-first (N=64, 3x224x224 -> 64 channels, fp16, F=16),
    both fold axes; the oracle checks sampled images, the whole output is checked for holes."""
    from paper_2601_11608_amd import workloads as wl

    layers, x, ws, bs = wl.make_config("c2")
    l = layers[0]
    xn = x.permute(0, 3, 1, 2).contiguous()
    wn = ws[0].permute(3, 2, 0, 1).contiguous()
    plan = fc.foldconv_plan_nchw(l.N, l.C_in, l.H, l.W, l.C_out, l.KH, l.KW, l.pad, l.F, axis_code(fc, axis), xn.dtype)
    print("nchw full size", axis, flush=True)
    y = run_nchw(fc, plan, xn, wn, bs[0], False).reshape(l.N, l.C_out, l.H, l.W)
    assert not bool(torch.isnan(y).any()), "unwritten output elements"
    images = [0, 40, 63]
    ref = oracle.conv_direct_nchw(f64(xn[images]), f64(wn), f64(bs[0]), 1, 1)
    assert rel_l2_per_image(f64(y[images]), ref) <= TOL["f16"]


def test_nchw_argument_errors(fc):
    with pytest.raises(fc.FoldconvError) as e:
        fc.foldconv_plan_nchw(1, 3, 30, 32, 8, 3, 3, 1, 4, fc.FOLD_H, torch.float16)     # 30 % 4
    assert e.value.status == -2
    with pytest.raises(fc.FoldconvError) as e:
        fc.foldconv_plan_nchw(1, 3, 32, 32, 8, 3, 3, 1, 4, 2, torch.float16)             # unknown axis
    assert e.value.status == -1
    plan = fc.foldconv_plan_nchw(1, 3, 32, 32, 8, 3, 3, 1, 4, fc.FOLD_H, torch.float16)
    x = torch.zeros(3 * 32 * 32, dtype=torch.float16, device="cuda")
    with pytest.raises(fc.FoldconvError) as e:
        fc.foldconv_fold_input_nchw(plan, x, x)                                          # in place is not possible
    assert e.value.status == -1
