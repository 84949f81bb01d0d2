"""Pins for the channels-first (NCHW / OIHW) part of the fp64 oracle and its
height-folding rewrite (paper: Introduction, height folding for NCHW).  As in
test_oracle_pins.py every check compares against something other than the
routine itself: the library's native NCHW convolution, the already pinned
NHWC oracle through explicit permutes, hand-worked values, closed forms and
brute-force index loops."""
import itertools

import numpy as np
import pytest
import torch


def rng(seed):
    return np.random.default_rng(seed)


CASES = [
    # N, C, H, W, Co, KH, KW, ph, pw, bias
    (1, 1, 5, 6, 1, 3, 3, 1, 1, False),
    (2, 3, 8, 7, 5, 3, 3, 1, 1, True),
    (1, 2, 12, 5, 4, 5, 1, 0, 0, True),    # K x 1, VALID: the setting of the paper's proof
    (2, 1, 20, 1, 3, 9, 1, 4, 0, False),   # Conv1d along H
    (1, 4, 8, 8, 2, 4, 2, 2, 1, True),     # even kernels, unequal pads
    (3, 2, 4, 5, 2, 1, 1, 0, 0, True),     # 1x1
    (1, 2, 6, 6, 3, 3, 3, 2, 2, True),     # more padding than 'same'
]


@pytest.mark.parametrize("N,C,H,W,Co,KH,KW,ph,pw,hb", CASES)
def test_conv_direct_nchw_pins(oracle, N, C, H, W, Co, KH, KW, ph, pw, hb):
    r = rng(7)
    x = r.standard_normal((N, C, H, W))
    w = r.standard_normal((Co, C, KH, KW))
    b = r.standard_normal(Co) if hb else None
    got = oracle.conv_direct_nchw(x, w, b, ph, pw)
    # the library's cross-correlation is natively NCHW / OIHW
    lib = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w),
                                     None if b is None else torch.from_numpy(b), stride=1, padding=(ph, pw)).numpy()
    assert got.shape == lib.shape
    assert np.allclose(got, lib, rtol=0, atol=1e-12)
    # the NHWC oracle (pinned on its own) through explicit permutes
    nhwc = oracle.conv_direct(x.transpose(0, 2, 3, 1), w.transpose(2, 3, 1, 0), b, ph, pw).transpose(0, 3, 1, 2)
    assert np.allclose(got, nhwc, rtol=0, atol=1e-12)
    relu = oracle.conv_direct_nchw(x, w, b, ph, pw, relu=True)
    assert np.array_equal(relu, np.maximum(got, 0.0))


def test_conv_nchw_hand_worked(oracle):
    # one channel, 3x2 image, 2x1 kernel along H, no padding:  y[h,w] = 1*x[h,w] + 10*x[h+1,w]
    x = np.array([[1., 2.], [3., 4.], [5., 6.]]).reshape(1, 1, 3, 2)
    w = np.array([1., 10.]).reshape(1, 1, 2, 1)
    y = oracle.conv_direct_nchw(x, w)
    assert np.array_equal(y.reshape(2, 2), np.array([[31., 42.], [53., 64.]]))
    # transposed operands or a flipped kernel would give [[13,24],[35,46]]
    # two input channels, distinct weights: catches a swapped C / Co axis
    x2 = np.stack([np.full((2, 2), 1.0), np.full((2, 2), 2.0)]).reshape(1, 2, 2, 2)
    w2 = np.array([[3.0, 5.0]]).reshape(1, 2, 1, 1)
    assert np.array_equal(oracle.conv_direct_nchw(x2, w2), np.full((1, 1, 2, 2), 13.0))


@pytest.mark.parametrize("N,C,H,W,F", [(1, 1, 8, 3, 4), (2, 3, 12, 2, 4), (1, 1, 32, 1, 32), (2, 5, 6, 3, 1), (1, 2, 6, 4, 6)])
def test_height_fold_definition(oracle, N, C, H, W, F):
    """xh[n, f*C+c, h', w] = x[n, c, F*h'+f, w] by brute-force loops, and as reshape + permute.
    Unlike the NHWC width fold this is NOT the identity on bytes unless F == 1."""
    x = rng(3).standard_normal((N, C, H, W))
    xh = oracle.fold_input_h_nchw(x, F)
    assert xh.shape == (N, F * C, H // F, W)
    for n, c, hp, f, wi in itertools.product(range(N), range(C), range(H // F), range(F), range(W)):
        assert xh[n, f * C + c, hp, wi] == x[n, c, F * hp + f, wi]
    assert np.array_equal(xh, x.reshape(N, C, H // F, F, W).transpose(0, 3, 1, 2, 4).reshape(N, F * C, H // F, W))
    if F > 1 and H // F > 1:
        assert not np.array_equal(xh.ravel(), x.ravel())
    # the NHWC width fold of the spatially transposed image holds the same numbers
    xw = oracle.fold_input(x.transpose(0, 3, 2, 1), F)            # [N, W, H/F, F*C]
    assert np.array_equal(xw.transpose(0, 3, 2, 1), xh)
    with pytest.raises(AssertionError):
        oracle.fold_input_h_nchw(rng(0).standard_normal((1, 1, 7, 2)), 2)


EXP = [(1, 1, 5, 1, 8, 0), (4, 3, 3, 3, 4, 1), (2, 2, 4, 2, 4, 2), (3, 1, 9, 1, 32, 4), (2, 3, 3, 2, 1, 1), (2, 2, 5, 3, 2, 2)]


@pytest.mark.parametrize("Co,C,KH,KW,F,p", EXP)
def test_height_expand_against_width_expand_and_structure(oracle, Co, C, KH, KW, F, p):
    w = rng(5).standard_normal((Co, C, KH, KW))
    wh = oracle.expand_filter_h_oihw(w, F, p)
    sh = oracle.folded_shapes(F, KH, p, F)
    assert wh.shape == (F * Co, F * C, sh["KWf"], KW)
    # element-wise definition by brute force (gather form, independent of the scatter loops)
    for g, co, f, c, dd, kw in itertools.product(range(F), range(Co), range(F), range(C), range(sh["KWf"]), range(KW)):
        kh = F * (dd + sh["d_min"]) + f - g + p
        want = w[co, c, kh, kw] if 0 <= kh < KH else 0.0
        assert wh[g * Co + co, f * C + c, dd, kw] == want
    # the pinned NHWC/HWIO expansion of the transposed kernel holds the same numbers:
    # HWIO of the transposed image is [KW][KH][C][Co]; its width-expanded form [KW][KHf][F*C][F*Co]
    we = oracle.expand_filter(w.transpose(3, 2, 1, 0), F, p)
    assert np.array_equal(we.transpose(3, 2, 1, 0), wh)
    # F*KH non-zero C x Co blocks per kw when the filter has no zero entries
    assert np.count_nonzero(wh) == F * KH * KW * C * Co


REWRITE = [
    # N, C, H, W, Co, KH, KW, ph, pw, F, bias
    (1, 1, 16, 3, 1, 5, 1, 0, 0, 8, True),     # the paper's K x 1 VALID proof setting, folded along H
    (2, 3, 12, 5, 4, 3, 3, 1, 1, 4, True),
    (1, 2, 8, 4, 3, 3, 3, 1, 1, 8, False),     # F == H
    (1, 1, 32, 2, 2, 9, 1, 4, 0, 16, True),
    (2, 2, 12, 3, 2, 4, 2, 2, 1, 4, False),    # even kernel: H_out = H + 1, ragged folded output
    (1, 3, 10, 4, 2, 3, 3, 0, 0, 5, True),     # VALID: H_out = 8, ragged
    (1, 2, 6, 6, 3, 3, 3, 1, 1, 1, True),      # F = 1
    (1, 1, 6, 3, 2, 7, 3, 3, 1, 2, False),     # KH > F
]


@pytest.mark.parametrize("N,C,H,W,Co,KH,KW,ph,pw,F,hb", REWRITE)
def test_height_rewrite_equals_direct(oracle, N, C, H, W, Co, KH, KW, ph, pw, F, hb):
    r = rng(11)
    x = r.standard_normal((N, C, H, W))
    w = r.standard_normal((Co, C, KH, KW))
    b = r.standard_normal(Co) if hb else None
    direct = oracle.conv_direct_nchw(x, w, b, ph, pw)
    y, parts = oracle.conv_rewrite_h_nchw(x, w, b, ph, pw, F, return_parts=True)
    assert y.shape == direct.shape
    assert np.allclose(y, direct, rtol=0, atol=1e-12)
    sh = parts["shapes"]
    assert parts["yh"].shape == (N, F * Co, sh["Wf_out"], W + 2 * pw - KW + 1)
    # and through the library, on the folded tensors with explicit asymmetric height padding
    top, bottom = sh["pad_left_f"], sh["pad_right_f"]
    xp = np.zeros((N, F * C, H // F + top + max(bottom, 0), W + 2 * pw))
    xp[:, :, top:top + H // F, pw:pw + W] = parts["xh"]
    bt = None if b is None else torch.from_numpy(np.tile(b, F))
    lib = torch.nn.functional.conv2d(torch.from_numpy(xp), torch.from_numpy(parts["wh"]), bt).numpy()
    assert np.allclose(parts["yh"], lib[:, :, :sh["Wf_out"], :], rtol=0, atol=1e-12)


def test_height_unfold_inverts_fold_and_crops(oracle):
    N, Co, H, W, F = 2, 3, 12, 4, 4
    y = rng(2).standard_normal((N, Co, H, W))
    yh = oracle.fold_input_h_nchw(y, F)
    assert np.array_equal(oracle.unfold_output_h_nchw(yh, F, Co, H), y)
    assert np.array_equal(oracle.unfold_output_h_nchw(yh, F, Co, H - 3), y[:, :, :H - 3, :])
