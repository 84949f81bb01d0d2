"""GPU parity of the folded convolution that writes its output channels-first in
the same launch (FLAG_OUT_NCHW), through the C ABI: bit-identical to the
two-step route (folded output, then the channels-first reconstruct) and within
the relative-L2 tolerance of the fp64 oracle."""
import numpy as np
import pytest
import torch

from helpers import TOL, TORCH_DT, f64, rel_l2_per_image

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


def prepare(fc, plan, x, w):
    s = plan.shapes
    dt = x.dtype
    w_exp = torch.empty(s.w_exp_bytes // s.elem_bytes, dtype=dt, device="cuda")
    fc.foldconv_expand_filter_oihw(plan, w.cuda(), w_exp)
    xf = torch.empty(x.numel(), dtype=dt, device="cuda")
    fc.foldconv_fold_input_nchw(plan, x.cuda(), xf)
    ws = torch.empty(max(int(s.workspace_bytes), 256), dtype=torch.uint8, device="cuda")
    return xf, w_exp, ws


def two_step(fc, plan, xf, w_exp, b, ws, flags):
    s = plan.shapes
    yf = torch.full((s.y_fold_bytes // s.elem_bytes,), float("nan"), dtype=xf.dtype, device="cuda")
    fc.foldconv_forward(plan, xf, w_exp, b, yf, ws, fc.FLAG_KEEP_FOLDED | flags)
    y = torch.full((s.y_bytes // s.elem_bytes,), float("nan"), dtype=xf.dtype, device="cuda")
    fc.foldconv_unfold_output_nchw(plan, yf, y)
    return y


def stage_fits(s):
    """Width fold: the rows of the channels-first input that a tile needs fit LDS beside the two output tiles
    (the library's rule, restated: 16-byte pieces, no tile across images, one piece per thread and tile)."""
    if s.W % 8 or (s.H_out * s.W_out_fold) % 32 or s.W_out_fold > s.W_fold:
        return False
    rows = (s.W_out_fold - 1 + 31) // s.W_out_fold + 1 + s.KH - 1
    halo = -s.d_min * s.C_fold + (s.d_max + 1) * s.C_fold - s.C_fold
    pitch = -(-(halo + s.W * s.C_in) * 2 // 16) * 16
    return rows * s.C_in * (s.W // 8) <= s.Co_fold and 2 * 32 * (s.Co_fold * 2 + 8) + 2 * rows * pitch <= 163840


def fused(fc, plan, xf, w_exp, b, ws, flags):
    s = plan.shapes
    y = torch.full((s.y_bytes // s.elem_bytes,), float("nan"), dtype=xf.dtype, device="cuda")
    fc.foldconv_forward(plan, xf, w_exp, b, y, ws, fc.FLAG_OUT_NCHW | flags)
    return y


# N, C, H, W, Co, KH, KW, pad, F, bias, relu
FUSED = [
    (2, 3, 32, 48, 64, 3, 3, 1, 16, True, True),      # headline structure: 16 waves per workgroup
    (3, 3, 5, 48, 64, 3, 3, 1, 16, True, False),      # 45 folded pixels: one full tile and a ragged one
    (1, 1, 24, 64, 32, 3, 3, 1, 8, False, True),      # 4 waves, several workgroups per compute unit
    (3, 1, 17, 96, 16, 3, 3, 1, 32, True, False),     # F = 32, C_out = 16
    (2, 2, 9, 40, 16, 1, 1, 0, 8, True, True),        # 1 x 1 kernel
    (1, 1, 12, 128, 12, 3, 3, 1, 16, True, False),    # C_out = 12: 64-column waves straddle slots
    (16, 3, 128, 128, 64, 3, 3, 1, 16, True, True),   # 512 tiles: every workgroup walks two
    (2, 2, 10, 64, 24, 2, 3, 1, 8, False, False),     # KH = 2: the guarded instance
    (70, 1, 1, 16, 8, 1, 1, 0, 16, True, False),      # one folded pixel per image: a tile spans 32 images
    (5, 1, 3, 32, 16, 3, 3, 1, 16, True, True),       # two folded pixels per row, three rows
    (1, 1, 300, 8, 64, 3, 1, 1, 8, False, False),     # one folded pixel per row, 3 x 1 kernel
    (2, 2, 11, 64, 24, 2, 3, 1, 8, False, True),      # KH = 2 (guarded instance) on a shape whose channels-first rows fit LDS
    (2, 2, 8, 64, 16, 1, 1, 0, 8, True, False),       # 1 x 1 kernel, the same; 2 waves
]


# Height folds (the plan is the transposed image's): N, C, H, W, Co, KH, KW, pad, F, bias, relu
FUSED_H = [
    (2, 3, 48, 32, 64, 3, 3, 1, 16, True, True),      # the headline structure, transposed: 16 waves, 3 folded columns
    (3, 3, 48, 40, 64, 3, 3, 1, 16, True, False),     # W = 40: a full row block of 32 and a ragged one of 8
    (1, 1, 64, 24, 32, 3, 3, 1, 8, False, True),      # 4 waves per workgroup
    (2, 2, 40, 16, 16, 1, 1, 0, 4, True, True),       # 1 x 1 kernel, F = 4 (a height fold needs no multiple of 8)
    (1, 1, 128, 8, 12, 3, 3, 1, 16, True, False),     # C_out = 12: 64-column waves straddle slots; one row block of 8
    (5, 3, 224, 64, 64, 3, 3, 1, 16, True, True),     # 14 folded columns per row block, tiles dealt over the XCDs
    (2, 2, 64, 25, 24, 3, 2, 0, 8, False, False),     # KW = 2 (the plan's KH): the guarded instance; VALID, W_out = 24, H_out = 62
    (2, 1, 32, 18, 16, 3, 3, 0, 8, True, False),      # VALID: H_out = 30 is not a multiple of F: the last slots are dropped; W_out = 16
    (3, 1, 16, 8, 8, 1, 1, 0, 16, True, False),       # one folded column, one row block
    # image wider than 64 columns and F*C_out a multiple of 128: quads of four tiles, 256-byte store runs
    (2, 3, 48, 136, 64, 3, 3, 1, 16, True, True),     # 16 waves; a full quad and one of 8 columns
    (1, 1, 64, 200, 32, 3, 3, 1, 8, False, True),     # 4 waves: two per tile group; 128 + 72 columns
    (2, 2, 40, 96, 16, 1, 1, 0, 8, True, True),       # 2 waves: one per tile group; 1 x 1 kernel; 96 columns: three tiles of a quad
    (1, 2, 32, 160, 32, 3, 3, 1, 4, True, False),     # F = 4: one slot per thread and pass
    (3, 3, 64, 138, 64, 3, 3, 0, 16, False, False),   # VALID: W_out = 136, H_out = 62: the last slots of the last folded column are dropped
]


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("case", FUSED + FUSED_H, ids=lambda c: "x".join(map(str, c[:9])))
def test_fused_nchw_output(fc, oracle, case, dt):
    N, C, H, W, Co, KH, KW, pad, F, hb, relu = case
    x = draw((N, C, H, W), dt, 41)
    w = (draw((Co, C, KH, KW), dt, 42) * (1.0 / np.sqrt(KH * KW * C))).to(TORCH_DT[dt])
    b = draw((Co,), dt, 43).cuda() if hb else None
    axis = fc.FOLD_H if case in FUSED_H else fc.FOLD_W
    plan = fc.foldconv_plan_nchw(N, C, H, W, Co, KH, KW, pad, F, axis, x.dtype)
    s = plan.shapes
    assert s.out_nchw_fused == 1, s.as_dict()
    print("fused nchw", "H" if axis == fc.FOLD_H else "W", case, dt, flush=True)
    xf, w_exp, ws = prepare(fc, plan, x, w)
    flags = fc.FLAG_RELU if relu else 0
    want = two_step(fc, plan, xf, w_exp, b, ws, flags)
    got = fused(fc, plan, xf, w_exp, b, ws, flags)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(got).any()), "unwritten output elements"
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    # the compact filter gives the same bytes
    cws = torch.empty(int(s.filter_compact_bytes), dtype=torch.uint8, device="cuda")
    # (the compact form is built from the HWIO filter of the plan's space: taps transposed for a height fold)
    w_hwio = w.permute(3, 2, 1, 0) if axis == fc.FOLD_H else w.permute(2, 3, 1, 0)
    fc.foldconv_pack_filter_compact(plan, w_hwio.contiguous().cuda(), cws)
    got_c = fused(fc, plan, xf, None, b, cws, flags | fc.FLAG_FILTER_COMPACT)
    torch.cuda.synchronize()
    assert torch.equal(got_c.view(torch.int16), want.view(torch.int16))
    # the channels-first input read in the same launch (no folded copy): the same bytes again.  Height folds
    # gather it element by element; width folds stage its rows through LDS where those fit
    xn = x.cuda().reshape(-1)
    if axis == fc.FOLD_H or stage_fits(s):
        got_in = fused(fc, plan, xn, w_exp, b, ws, flags | fc.FLAG_IN_NCHW)
        got_in_c = fused(fc, plan, xn, None, b, cws, flags | fc.FLAG_IN_NCHW | fc.FLAG_FILTER_COMPACT)
        torch.cuda.synchronize()
        assert not bool(torch.isnan(got_in).any()), "unwritten output elements"
        assert torch.equal(got_in.view(torch.int16), want.view(torch.int16))
        assert torch.equal(got_in_c.view(torch.int16), want.view(torch.int16))
    else:
        with pytest.raises(fc.FoldconvError) as e:
            fused(fc, plan, xn, w_exp, b, ws, flags | fc.FLAG_IN_NCHW)
        assert e.value.status == -3
    if N * Co * H * W <= 1 << 21:
        ph, pw = oracle.axis_pads(KH, KW, pad)
        ref = oracle.conv_direct_nchw(f64(x), f64(w), None if b is None else f64(b.cpu()), ph, pw, relu)
        assert rel_l2_per_image(f64(got.cpu()).reshape(ref.shape), ref) <= TOL[dt]


@pytest.mark.parametrize("chunk", range(4))
def test_fused_nchw_random_geometries(fc, chunk):
    """Seeded random shapes that the channels-first kernel serves, both folds: the one-launch call (channels-first
    input and output) and the fused-output call write the bytes of the two-step route (which the other tests tie to
    the oracle).  Shapes are drawn so that pairs and quads of tiles, the staged and the gathered input read, ragged
    tiles and images that are not a whole number of tiles all occur."""
    rng = np.random.RandomState(4100 + chunk)
    ran, one_launch, two_launch = 0, 0, 0
    tries = 0
    while ran < 12 and tries < 400:
        tries += 1
        axis = fc.FOLD_H if rng.rand() < 0.5 else fc.FOLD_W
        N, C = int(rng.randint(1, 4)), int(rng.choice([1, 2, 3, 4]))
        Co = int(rng.choice([8, 16, 32, 64]))
        F = int(rng.choice([4, 8, 16] if axis == fc.FOLD_H else [8, 16, 32]))
        k = int(rng.choice([1, 3]))
        KH, KW, pad = k, k, k // 2
        # the folded axis is a multiple of F, the other one a multiple of 8
        a_fold = F * int(rng.randint(1, 9))
        a_other = 8 * int(rng.randint(1, 26))
        H, W = (a_fold, a_other) if axis == fc.FOLD_H else (a_other, a_fold)
        if F * Co > 1024 or (F * Co) % 64:
            continue
        plan = fc.foldconv_plan_nchw(N, C, H, W, Co, KH, KW, pad, F, axis, torch.float16)
        s = plan.shapes
        if not s.out_nchw_fused:
            continue
        dt = "f16" if rng.rand() < 0.5 else "bf16"
        if dt == "bf16":
            plan = fc.foldconv_plan_nchw(N, C, H, W, Co, KH, KW, pad, F, axis, torch.bfloat16)
            s = plan.shapes
        seed = int(rng.randint(1 << 30))
        x = draw((N, C, H, W), dt, seed)
        w = (draw((Co, C, KH, KW), dt, seed + 1) * (1.0 / np.sqrt(KH * KW * C))).to(TORCH_DT[dt])
        b = draw((Co,), dt, seed + 2).cuda() if rng.rand() < 0.7 else None
        flags = fc.FLAG_RELU if rng.rand() < 0.5 else 0
        print("random fused nchw", "H" if axis == fc.FOLD_H else "W", (N, C, H, W, Co, KH, KW, pad, F), dt, flush=True)
        xf, w_exp, ws = prepare(fc, plan, x, w)
        want = two_step(fc, plan, xf, w_exp, b, ws, flags)
        got = fused(fc, plan, xf, w_exp, b, ws, flags)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), want.view(torch.int16))
        try:
            got_in = fused(fc, plan, x.cuda().reshape(-1), w_exp, b, ws, flags | fc.FLAG_IN_NCHW)
            torch.cuda.synchronize()
            assert torch.equal(got_in.view(torch.int16), want.view(torch.int16))
            one_launch += 1
        except fc.FoldconvError as e:
            assert e.status == -3 and axis == fc.FOLD_W and not stage_fits(s)
            two_launch += 1
        ran += 1
    assert ran == 12 and one_launch >= 6


@pytest.mark.parametrize("axis", ["W", "H"])
def test_fused_nchw_headline_layer_full_size(fc, oracle, axis):
    """The headline layer (N=64, 3x224x224 -> 64 channels, fp16, F=16) written channels-first in one
    launch: identical to the two-step route everywhere, sampled images against the oracle."""
    from paper_2601_11608_amd import workloads as wl

    layers, x, wts, bs = wl.make_config("c2")
    l = layers[0]
    xn = x.permute(0, 3, 1, 2).contiguous()
    wn = wts[0].permute(3, 2, 0, 1).contiguous()
    plan = fc.foldconv_plan_nchw(l.N, l.C_in, l.H, l.W, l.C_out, l.KH, l.KW, l.pad, l.F,
                                 fc.FOLD_W if axis == "W" else fc.FOLD_H, xn.dtype)
    assert plan.shapes.out_nchw_fused == 1
    print("fused nchw full size, fold", axis, flush=True)
    xf, w_exp, ws = prepare(fc, plan, xn, wn)
    b = bs[0].cuda()
    want = two_step(fc, plan, xf, w_exp, b, ws, 0)
    got = fused(fc, plan, xf, w_exp, b, ws, 0)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    got_in = fused(fc, plan, xn.cuda().reshape(-1), w_exp, b, ws, fc.FLAG_IN_NCHW)      # channels-first on both sides
    torch.cuda.synchronize()
    assert torch.equal(got_in.view(torch.int16), want.view(torch.int16))
    y = got.cpu().reshape(l.N, l.C_out, l.H, l.W)
    images = [0, 29, 63]
    ref = oracle.conv_direct_nchw(f64(xn[images]), f64(wn), f64(bs[0]), 1, 1)
    assert rel_l2_per_image(f64(y[images]), ref) <= TOL["f16"]


@pytest.mark.parametrize("axis", ["W", "H"])
def test_channels_first_layer_runner(fc, oracle, axis):
    """runner.ChannelsFirstLayer takes the fused route where the plan offers it (both folds here); both match
    the oracle."""
    from paper_2601_11608_amd import workloads as wl
    from paper_2601_11608_amd.runner import ChannelsFirstLayer

    l = wl.Layer("t", 2, 32, 48, 3, 64, 3, 3, 1, 16, "f16", True, "normal", relu=True)
    x = draw((l.N, l.C_in, l.H, l.W), "f16", 51)
    w = (draw((l.C_out, l.C_in, 3, 3), "f16", 52) * (1.0 / np.sqrt(27))).to(torch.float16)
    b = draw((l.C_out,), "f16", 53)
    L = ChannelsFirstLayer(l, w, b, fc.FOLD_W if axis == "W" else fc.FOLD_H)
    assert L.fused
    y = L.forward(x.cuda(), L.new_output())
    torch.cuda.synchronize()
    ref = oracle.conv_direct_nchw(f64(x), f64(w), f64(b), 1, 1, True)
    assert tuple(y.shape) == ref.shape
    assert rel_l2_per_image(f64(y.cpu()), ref) <= TOL["f16"]


def test_fused_nchw_under_graph_capture(fc):
    """The library allocates nothing and never synchronises, so the call can be captured; every replay
    (with eager work and synchronisations between them) equals the eager result."""
    dt = torch.float16
    plan = fc.foldconv_plan_nchw(4, 3, 40, 64, 64, 3, 3, 1, 16, fc.FOLD_W, dt)
    s = plan.shapes
    x = draw((4, 3, 40, 64), "f16", 71)
    w = (draw((64, 3, 3, 3), "f16", 72) * 0.2).to(dt)
    b = draw((64,), "f16", 73).cuda()
    xf, w_exp, ws = prepare(fc, plan, x, w)
    fc.foldconv_pack_filter(plan, w_exp, ws)
    flags = fc.FLAG_OUT_NCHW | fc.FLAG_FILTER_PACKED | fc.FLAG_RELU
    y = torch.zeros(s.y_bytes // 2, dtype=dt, device="cuda")
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=st):
        fc.foldconv_forward(plan, xf, w_exp, b, y, ws, flags, stream=st)
    want = torch.zeros_like(y)
    fc.foldconv_forward(plan, xf, w_exp, b, want, ws, flags)
    torch.cuda.synchronize()
    assert float(want.float().abs().sum()) > 0
    for _ in range(3):
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), want.view(torch.int16))


def test_fused_nchw_refusals(fc):
    dt = torch.float16
    # geometries the fused kernel does not serve report it in the plan and are refused by the call
    for args, axis in [((1, 3, 8, 16, 4, 3, 3, 1, 16), fc.FOLD_W),      # one wave would span all 16 slots: K too wide
                       ((1, 12, 16, 32, 16, 3, 3, 1, 8), fc.FOLD_W),    # C_in = 12: five K-steps per kh
                       ((1, 3, 16, 30, 64, 3, 3, 0, 2), fc.FOLD_W),     # F not a multiple of 8
                       ((1, 3, 16, 32, 64, 3, 3, 0, 16), fc.FOLD_W),    # VALID: W_out = 30 is not F * W'_out
                       ((2, 3, 32, 44, 64, 3, 3, 1, 16), fc.FOLD_H),    # height fold, W_out = 44 not a multiple of 8
                       ((1, 12, 32, 16, 16, 3, 3, 1, 8), fc.FOLD_H)]:   # height fold, C_in = 12: five K-steps per kh
        plan = fc.foldconv_plan_nchw(*args, axis, dt)
        s = plan.shapes
        assert s.out_nchw_fused == 0, args
        x = torch.zeros(s.x_bytes // 2, dtype=dt, device="cuda")
        w = torch.zeros(s.w_exp_bytes // 2, dtype=dt, device="cuda")
        y = torch.zeros(max(s.y_bytes, s.y_fold_bytes) // 2, dtype=dt, device="cuda")
        ws = torch.empty(max(int(s.workspace_bytes), 256), dtype=torch.uint8, device="cuda")
        with pytest.raises(fc.FoldconvError) as e:
            fc.foldconv_forward(plan, x, w, None, y, ws, fc.FLAG_OUT_NCHW)
        assert e.value.status == -3
    plan = fc.foldconv_plan_nchw(2, 3, 32, 48, 64, 3, 3, 1, 16, fc.FOLD_W, dt)
    s = plan.shapes
    x = torch.zeros(s.x_bytes // 2, dtype=dt, device="cuda")
    w = torch.zeros(s.w_exp_bytes // 2, dtype=dt, device="cuda")
    y = torch.zeros(s.y_bytes // 2, dtype=dt, device="cuda")
    ws = torch.empty(int(s.workspace_bytes), dtype=torch.uint8, device="cuda")
    with pytest.raises(fc.FoldconvError) as e:
        fc.foldconv_forward(plan, x, w, None, y, ws, fc.FLAG_OUT_NCHW | fc.FLAG_KEEP_FOLDED)
    assert e.value.status == -1
    # a channels-first input is only read by the kernel that also writes channels-first
    with pytest.raises(fc.FoldconvError) as e:
        fc.foldconv_forward(plan, x, w, None, y, ws, fc.FLAG_IN_NCHW)
    assert e.value.status == -1
    # the dense walk needs more K-steps per kh than the fused kernel holds
    with pytest.raises(fc.FoldconvError) as e:
        fc.foldconv_forward(plan, x, w, None, y, ws, fc.FLAG_OUT_NCHW | fc.FLAG_DENSE_K)
    assert e.value.status == -3
