"""foldconv_forward_static (the entry point for callers that cannot allocate: the packed filter
lives in a device array inside the library) against foldconv_forward with a caller workspace:
same kernels, so the outputs must be identical bit for bit, call after call, also when a later
call uses less of the shared array than the one before it."""
import numpy as np
import pytest
import torch

from helpers import TORCH_DT, bits

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


def both_routes(fc, case, dt, seed, flags=0):
    N, H, W, C, Co, KH, KW, pad, F, hb, relu = case
    x = draw((N, H, W, C), dt, seed).cuda()
    w = (draw((KH, KW, C, Co), dt, seed + 1) * (1.0 / np.sqrt(KH * KW * C))).to(TORCH_DT[dt]).cuda()
    b = draw((Co,), dt, seed + 2).cuda() if hb else None
    plan = fc.foldconv_plan(N, H, W, C, Co, KH, KW, pad, F, x.dtype)
    s = plan.shapes
    assert s.workspace_bytes <= fc.STATIC_SCRATCH_BYTES
    flags |= fc.FLAG_RELU if relu else 0
    w_exp = torch.empty(s.w_exp_bytes // s.elem_bytes, dtype=x.dtype, device="cuda")
    fc.foldconv_expand_filter(plan, w, w_exp)
    ws = torch.empty(max(int(s.workspace_bytes), 256), dtype=torch.uint8, device="cuda")
    shape = (s.N, s.H_out, s.W_out_fold, s.Co_fold) if flags & fc.FLAG_KEEP_FOLDED else (s.N, s.H_out, s.W_out, s.C_out)
    y_ws = torch.full(shape, float("nan"), dtype=x.dtype, device="cuda")
    y_st = torch.full(shape, float("nan"), dtype=x.dtype, device="cuda")
    fc.foldconv_forward(plan, x, w_exp, b, y_ws, ws, flags)
    fc.foldconv_forward_static(plan, x, w_exp, b, y_st, flags)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(y_ws).any())
    return plan, y_ws.cpu(), y_st.cpu()


# N, H, W, C, Co, KH, KW, pad, F, bias, relu
BIG = (2, 24, 56, 68, 132, 3, 3, 1, 4, True, True)      # tiled kernel, 2.6 MB of packed filter
SMALL = (3, 7, 32, 3, 64, 3, 3, 1, 16, True, True)      # streaming kernel, 0.9 MB: less than the call before
TINY = (1, 6, 12, 2, 3, 3, 3, 0, 4, True, False)        # ragged reconstruct, 5 KB
GATHER = (2, 5, 7, 3, 3, 3, 3, 1, 1, True, True)        # element-gather kernel: no scratch at all


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_static_scratch_matches_caller_workspace_call_after_call(fc, dt):
    for i, case in enumerate((BIG, SMALL, BIG, TINY, GATHER, SMALL)):
        print("static scratch", dt, i, case, flush=True)
        plan, y_ws, y_st = both_routes(fc, case, dt, 300 + 10 * i)
        assert np.array_equal(bits(y_ws), bits(y_st)), (i, case)
    for extra in (fc.FLAG_DENSE_K, fc.FLAG_KEEP_FOLDED):
        plan, y_ws, y_st = both_routes(fc, SMALL, dt, 400, extra)
        assert np.array_equal(bits(y_ws), bits(y_st)), extra


def test_static_scratch_fp32(fc):
    plan, y_ws, y_st = both_routes(fc, (1, 32, 32, 3, 16, 3, 3, 1, 8, False, False), "f32", 500)
    assert np.array_equal(bits(y_ws), bits(y_st))


def test_static_scratch_rejects_what_it_cannot_serve(fc):
    plan = fc.foldconv_plan(*SMALL[:9], torch.float16)
    s = plan.shapes
    t = torch.zeros(max(s.x_bytes, s.y_bytes, s.w_exp_bytes) // 2, dtype=torch.float16, device="cuda")
    for flag in (fc.FLAG_FILTER_PACKED, fc.FLAG_FILTER_COMPACT):
        with pytest.raises(fc.FoldconvError) as e:
            fc.foldconv_forward_static(plan, t, t, None, t, flag)
        assert e.value.status == -1
    big = fc.foldconv_plan(1, 8, 64, 132, 256, 3, 3, 1, 16, torch.float16)       # 78 MB of packed filter
    assert big.shapes.workspace_bytes > fc.STATIC_SCRATCH_BYTES
    with pytest.raises(fc.FoldconvError) as e:     # raw pointers: the size is refused by the library, not the binding
        fc.foldconv_forward_static(big, t.data_ptr(), t.data_ptr(), None, t.data_ptr(), 0)
    assert e.value.status == -6
