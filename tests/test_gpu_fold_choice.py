"""The fold-factor cost model on the GPU: for the benchmark layers (at a reduced batch; the choice is
made for the full batch) and a few mid-network shapes, the factor foldconv_choose_fold returns is
planned, run through the C ABI and checked against the fp64 oracle, and so is every other legal
power-of-two factor (so that whatever a recalibrated model may pick is known to compute the same
convolution).  paper: "F is chosen to align with Tensor core tile sizes"; the lightweight cost model of
"Compiler-Level Realization in MLIR"."""
import numpy as np
import pytest
import torch

from helpers import TOL, TORCH_DT, assert_elementwise, f64, rel_l2_per_image

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fc():
    import paper_2601_11608_amd as fc

    fc.load_library()
    assert torch.cuda.is_available()
    return fc


# name, full batch N, run batch, H, W, C_in, C_out, KH, KW, pad, dtype, bias, relu
LAYERS = [
    ("c1", 1, 1, 32, 32, 3, 16, 3, 3, 1, "f32", False, False),
    ("c2", 64, 2, 224, 224, 3, 64, 3, 3, 1, "f16", True, False),
    ("c2_f32", 64, 2, 224, 224, 3, 64, 3, 3, 1, "f32", True, False),
    ("c3", 32, 2, 112, 112, 12, 48, 3, 3, 1, "bf16", False, False),
    ("c4", 16, 2, 1, 16000, 1, 64, 1, 9, 4, "f16", False, False),
    ("c5_L1", 32, 2, 112, 112, 3, 20, 3, 3, 1, "bf16", False, True),
    ("c5_L2", 32, 2, 112, 112, 20, 36, 3, 3, 1, "bf16", False, True),
    ("c5_L3", 32, 1, 112, 112, 36, 68, 3, 3, 1, "bf16", False, True),
    ("c5_L4", 32, 1, 112, 112, 68, 132, 3, 3, 1, "bf16", False, True),
    ("c5_L5", 32, 1, 112, 112, 132, 256, 3, 3, 1, "bf16", False, False),
    ("mid 56x56 24->96", 16, 2, 56, 56, 24, 96, 3, 3, 1, "f16", True, True),
    ("mid 28x28 40->80 5x5", 16, 2, 28, 28, 40, 80, 5, 5, 2, "bf16", True, False),
    ("mid 56x56 6->32 1x1", 8, 2, 56, 56, 6, 32, 1, 1, 0, "f16", False, False),
    ("mid 64x96 10->24 3x1", 8, 2, 64, 96, 10, 24, 3, 1, 1, "bf16", True, True),
]


def draw(shape, dt, seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return torch.randn(shape, generator=g).to(TORCH_DT[dt])


@pytest.mark.parametrize("case", LAYERS, ids=lambda c: c[0].replace(" ", "_"))
def test_chosen_fold_factor_runs_and_matches_oracle(fc, oracle, case):
    name, N_full, N, H, W, C, Co, KH, KW, pad, dt, hb, relu = case
    pick = fc.foldconv_choose_fold(N_full, H, W, C, Co, KH, KW, pad, TORCH_DT[dt])
    assert pick >= 1 and W % pick == 0 and pick & (pick - 1) == 0
    x = draw((N, H, W, C), dt, 71)
    w = (draw((KH, KW, C, Co), dt, 72) * (1.0 / np.sqrt(KH * KW * C))).to(TORCH_DT[dt])
    b = draw((Co,), dt, 73) if hb else None
    ph, pw = oracle.axis_pads(KH, KW, pad)
    xf, wf, bf = f64(x), f64(w), None if b is None else f64(b)
    ref = oracle.conv_direct(xf, wf, bf, ph, pw, relu)
    S = oracle.conv_direct(np.abs(xf), np.abs(wf), None if bf is None else np.abs(bf), ph, pw, False)
    xd, wd, bd = x.cuda(), w.cuda(), None if b is None else b.cuda()
    factors = [F for F in (1, 2, 4, 8, 16, 32, 64) if W % F == 0]
    assert pick in factors
    for F in [pick] + [F for F in factors if F != pick]:
        plan = fc.foldconv_plan(N, H, W, C, Co, KH, KW, pad, F, x.dtype)
        s = plan.shapes
        if s.w_exp_bytes > (256 << 20):
            continue
        print("fold choice", name, "F", F, "(model pick)" if F == pick else "", "kernel", s.conv_kernel, flush=True)
        w_exp = torch.empty(s.w_exp_bytes // s.elem_bytes, dtype=x.dtype, device="cuda")
        fc.foldconv_expand_filter(plan, wd, w_exp)
        ws = torch.empty(max(int(s.workspace_bytes), 256), dtype=torch.uint8, device="cuda")
        y = torch.full((N, s.H_out, s.W_out, Co), float("nan"), dtype=x.dtype, device="cuda")
        fc.foldconv_fold_input(plan, xd, xd)
        fc.foldconv_forward(plan, xd, w_exp, bd, y, ws, fc.FLAG_RELU if relu else 0)
        torch.cuda.synchronize()
        got = f64(y)
        assert not np.isnan(got).any(), (name, F)
        assert rel_l2_per_image(got, ref) <= TOL[dt], (name, F)
        assert_elementwise(got, ref, S, KH * KW * C, dt, "%s F=%d" % (name, F))
        del w_exp, ws, y
