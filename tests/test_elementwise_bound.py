"""CPU checks of the element-wise bound the GPU parity tests use: the grid spacing it assumes is
the output types' real spacing, a correctly rounded fp32-accumulated result always passes, and a
planted mistake in the oracle's arithmetic (a dropped tap, a shifted tap) is caught by it even
where the per-image relative L2 tolerance lets it through."""
import numpy as np
import pytest
import torch

from helpers import (TOL, TORCH_DT, assert_elementwise, assert_same_to_rounding, f64, rel_l2_per_image, ulp_out)


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
def test_spacing_is_the_types_spacing(dt):
    t = TORCH_DT[dt]
    tiny = {"f16": 2.0 ** -24, "bf16": 2.0 ** -133, "f32": 2.0 ** -149}[dt]
    for v in (1.0, 1.5, 0.75, 3.0e-3, 1000.0, 6.0e-5, 2.0 ** -14, 2.0 ** -15, tiny, 3 * tiny):
        a = torch.tensor([v], dtype=torch.float64).to(t)
        nxt = torch.nextafter(a.float(), torch.tensor([float("inf")])).to(torch.float64) if dt == "f32" else None
        if dt == "f32":
            gap = float(nxt[0] - a.double()[0])
        else:
            bits = a.view(torch.int16) + 1
            gap = float(bits.view(t).double()[0] - a.double()[0])
        assert ulp_out(np.array([float(a.double()[0])]), dt)[0] == gap, v


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_a_correct_result_passes_and_planted_mistakes_fail(oracle, dt):
    g = torch.Generator(device="cpu")
    g.manual_seed(5)
    N, H, W, C, Co, KH, KW = 2, 12, 512, 3, 16, 3, 3
    x = torch.randn((N, H, W, C), generator=g).to(TORCH_DT[dt])
    w = (torch.randn((KH, KW, C, Co), generator=g) / np.sqrt(KH * KW * C)).to(TORCH_DT[dt])
    b = (torch.rand((Co,), generator=g) * 0.2 - 0.1).to(TORCH_DT[dt])
    xf, wf, bf = f64(x), f64(w), f64(b)
    ref = oracle.conv_direct(xf, wf, bf, 1, 1, False)
    S = oracle.conv_direct(np.abs(xf), np.abs(wf), np.abs(bf), 1, 1, False)
    K = KH * KW * C
    # a stand-in for the device arithmetic: fp32 accumulation (library routine), one rounding
    y32 = torch.nn.functional.conv2d(x.float().permute(0, 3, 1, 2), w.float().permute(3, 2, 0, 1), b.float(), padding=1)
    y = f64(y32.permute(0, 2, 3, 1).to(TORCH_DT[dt]))
    assert assert_elementwise(y, ref, S, K, dt, "fp32 accumulate") <= 1.0
    assert_same_to_rounding(y, y, S, K, dt)
    # planted in the oracle's inputs: one tap (kh=0, kw=2, c=1) of one output channel is missing in the
    # top rows of one column near the border (a wrong band edge): invisible to the relative L2 norm,
    # caught element by element
    w_bad = wf.copy()
    w_bad[0, 2, 1, 0] = 0.0
    bad = oracle.conv_direct(xf, w_bad, bf, 1, 1, False)
    y_bad = y.copy()
    y_bad[:, :3, W - 2, 0] = bad[:, :3, W - 2, 0]
    assert rel_l2_per_image(y_bad, ref) <= TOL[dt]
    with pytest.raises(AssertionError):
        assert_elementwise(y_bad, ref, S, K, dt, "dropped tap")
    with pytest.raises(AssertionError):
        assert_same_to_rounding(y, y_bad, S, K, dt, "dropped tap")
    # one output channel of one pixel two spacings off
    y_off = y.copy()
    y_off[1, 5, 7, 3] += 2.0 * ulp_out(y_off[1, 5, 7, 3], dt)
    with pytest.raises(AssertionError):
        assert_elementwise(y_off, ref, S, K, dt, "two spacings off")
