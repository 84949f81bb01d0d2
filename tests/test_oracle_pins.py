"""Pins for the fp64 CPU oracle: every check here compares the oracle with
something other than itself -- a library routine, an independent
formulation, a hand-worked value, a closed form or brute force -- chosen so
that a plausible slip (flipped kernel, dropped bias, transposed operand,
wrong pad sign, off-by-one in the fold) fails at least one of them."""
import itertools
import json
import os

import numpy as np
import pytest
import torch

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------------------
# direct convolution
# ----------------------------------------------------------------------------
def torch_conv(x, w, b, ph, pw, relu=False):
    """Library fp64 cross-correlation (NCHW/OIHW) as a second opinion."""
    xt = torch.from_numpy(np.ascontiguousarray(x)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(np.ascontiguousarray(w)).permute(3, 2, 0, 1)
    bt = None if b is None else torch.from_numpy(np.ascontiguousarray(b))
    y = torch.nn.functional.conv2d(xt, wt, bt, stride=1, padding=(ph, pw))
    if relu:
        y = torch.relu(y)
    return y.permute(0, 2, 3, 1).contiguous().numpy()


def einsum_conv(x, w, b, ph, pw):
    """Independent formulation: explicit zero-padded array + shifted views."""
    N, H, W, C = x.shape
    KH, KW, _, Co = w.shape
    xp = np.zeros((N, H + 2 * ph, W + 2 * pw, C))
    xp[:, ph:ph + H, pw:pw + W, :] = x
    Ho, Wo = H + 2 * ph - KH + 1, W + 2 * pw - KW + 1
    y = np.zeros((N, Ho, Wo, Co))
    for kh in range(KH):
        for kw in range(KW):
            y += np.einsum("nhwc,co->nhwo", xp[:, kh:kh + Ho, kw:kw + Wo, :], w[kh, kw])
    if b is not None:
        y = y + b
    return y


CONV_CASES = [
    # N, H, W, C, Co, KH, KW, ph, pw, bias
    (1, 5, 6, 1, 1, 3, 3, 1, 1, False),
    (2, 7, 8, 3, 5, 3, 3, 1, 1, True),
    (1, 6, 9, 2, 4, 5, 1, 0, 0, True),     # K x 1, VALID: the paper's proof setting
    (2, 1, 20, 1, 3, 1, 9, 0, 4, False),   # Conv1d as H = KH = 1
    (1, 8, 8, 4, 2, 2, 4, 1, 2, True),     # even kernels, unequal pads
    (1, 4, 5, 3, 3, 3, 3, 0, 0, False),    # VALID 3x3
    (3, 5, 4, 2, 2, 1, 1, 0, 0, True),     # 1x1 (GEMM as 1x1 conv)
    (1, 3, 3, 2, 3, 3, 3, 2, 2, True),     # pad larger than needed for 'same'
]


def pins_pass(conv_fn):
    """Run the value pins against ``conv_fn(x, w, b, ph, pw, relu)``.
    Returns the list of pins that failed (empty list == all pass)."""
    bad = []
    # (a) hand-worked 1-D: x=[1,2,3,4], w=[1,1,1], p=1 -> [3,6,9,7]
    x = np.array([1., 2, 3, 4]).reshape(1, 1, 4, 1)
    w = np.ones((1, 3, 1, 1))
    if not np.array_equal(conv_fn(x, w, None, 0, 1, False).ravel(), [3, 6, 9, 7]):
        bad.append("hand_1d_box")
    # (b) one-sided tap: w=[1,0,0] reads the LEFT neighbour (cross-correlation,
    #     no flip): y[w] = x[w-1] -> [0,1,2,3]
    w = np.array([1., 0, 0]).reshape(1, 3, 1, 1)
    if not np.array_equal(conv_fn(x, w, None, 0, 1, False).ravel(), [0, 1, 2, 3]):
        bad.append("hand_1d_left_tap")
    # (c) vertical one-sided tap on a 3x1 image column: w=[0,0,1]^T reads below
    xc = np.array([1., 2, 3]).reshape(1, 3, 1, 1)
    w = np.array([0., 0, 1]).reshape(3, 1, 1, 1)
    if not np.array_equal(conv_fn(xc, w, None, 1, 0, False).ravel(), [2, 3, 0]):
        bad.append("hand_vertical_tap")
    # (d) 3x3 ones on 3x3 ones, pad 1 -> neighbour counts
    x = np.ones((1, 3, 3, 1))
    w = np.ones((3, 3, 1, 1))
    if not np.array_equal(conv_fn(x, w, None, 1, 1, False)[0, :, :, 0],
                          [[4, 6, 4], [6, 9, 6], [4, 6, 4]]):
        bad.append("hand_2d_counts")
    # (e) channel mixing is c -> co, not co -> c: x has C=2, w maps channel 0
    #     to output 1 only with weight 5, channel 1 to output 0 with weight 7
    x = np.array([2., 3]).reshape(1, 1, 1, 2)
    w = np.zeros((1, 1, 2, 2)); w[0, 0, 0, 1] = 5; w[0, 0, 1, 0] = 7
    if not np.array_equal(conv_fn(x, w, None, 0, 0, False).ravel(), [21, 10]):
        bad.append("hand_channel_mix")
    # (f) bias only: w = 0 -> y == b everywhere; relu clamps negatives
    x = rng(0).standard_normal((2, 4, 5, 3))
    w = np.zeros((3, 3, 3, 2)); b = np.array([0.5, -1.25])
    y = conv_fn(x, w, b, 1, 1, False)
    if not (np.all(y[..., 0] == 0.5) and np.all(y[..., 1] == -1.25)):
        bad.append("bias_only")
    y = conv_fn(x, w, b, 1, 1, True)
    if not (np.all(y[..., 0] == 0.5) and np.all(y[..., 1] == 0.0)):
        bad.append("bias_relu")
    # (g) delta filter at the centre with 'same' padding is the identity
    x = rng(1).standard_normal((1, 5, 6, 2))
    w = np.zeros((3, 3, 2, 2)); w[1, 1, 0, 0] = 1; w[1, 1, 1, 1] = 1
    if not np.array_equal(conv_fn(x, w, None, 1, 1, False), x):
        bad.append("delta_identity")
    # (h) library routine and independent formulation on random cases
    for i, (N, H, W, C, Co, KH, KW, ph, pw, hb) in enumerate(CONV_CASES):
        r = rng(100 + i)
        x = r.standard_normal((N, H, W, C)); w = r.standard_normal((KH, KW, C, Co))
        b = r.standard_normal(Co) if hb else None
        y = conv_fn(x, w, b, ph, pw, False)
        yt = torch_conv(x, w, b, ph, pw)
        ye = einsum_conv(x, w, b, ph, pw)
        if y.shape != yt.shape or not np.allclose(y, yt, rtol=0, atol=1e-12):
            bad.append("torch_case_%d" % i)
        if y.shape != ye.shape or not np.allclose(y, ye, rtol=0, atol=1e-12):
            bad.append("einsum_case_%d" % i)
        yr = conv_fn(x, w, b, ph, pw, True)
        if not np.allclose(yr, torch_conv(x, w, b, ph, pw, relu=True), rtol=0, atol=1e-12):
            bad.append("torch_relu_case_%d" % i)
    return bad


def test_conv_direct_pins(oracle):
    assert pins_pass(lambda x, w, b, ph, pw, relu: oracle.conv_direct(x, w, b, ph, pw, relu)) == []


def _mutant(kind):
    """Pure-numpy convolutions with one planted mistake each."""
    def fn(x, w, b, ph, pw, relu):
        if kind == "flip_w":
            w2 = w[:, ::-1]
        elif kind == "flip_h":
            w2 = w[::-1]
        elif kind == "swap_cin_cout" and w.shape[2] == w.shape[3]:
            w2 = np.swapaxes(w, 2, 3)
        else:
            w2 = w
        bb = None if kind == "drop_bias" else b
        y = einsum_conv(x, w2, bb, ph, pw)
        if kind == "pad_sign":  # shifts the window the wrong way
            y = np.roll(y, 1, axis=2) if pw else y
        if kind == "relu_abs":
            y = np.abs(y) if relu else y
        elif relu:
            y = np.maximum(y, 0)
        return y
    return fn


@pytest.mark.parametrize("kind", ["flip_w", "flip_h", "swap_cin_cout", "drop_bias", "pad_sign", "relu_abs"])
def test_pins_catch_planted_mistakes(kind):
    assert pins_pass(_mutant(kind)) != [], "pins are blind to mistake %s" % kind


def test_pins_accept_correct_numpy():
    assert pins_pass(_mutant("none")) == []


# ----------------------------------------------------------------------------
# fold / unfold
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("N,H,W,C,F", [(1, 3, 8, 1, 4), (2, 2, 12, 3, 4), (1, 1, 32, 1, 32), (2, 3, 6, 5, 1), (1, 2, 6, 2, 6)])
def test_fold_is_reshape_and_offset_identity(oracle, N, H, W, C, F):
    x = rng(5).standard_normal((N, H, W, C))
    xf = oracle.fold_input(x, F)
    assert xf.shape == (N, H, W // F, F * C)
    # the appendix listing folds with a plain reshape
    assert np.array_equal(xf, x.reshape(N, H, W // F, F * C))
    # closed form: equal linear offsets in contiguous NHWC
    assert np.array_equal(xf.ravel(), x.ravel())
    # element-wise definition X'(h, w', f) = X(h, F w' + f) on probes
    for (n, h, wp, f, c) in itertools.product(range(N), range(H), range(W // F), range(F), range(C)):
        assert xf[n, h, wp, f * C + c] == x[n, h, F * wp + f, c]


def test_fold_rejects_indivisible_width(oracle):
    with pytest.raises(AssertionError):
        oracle.fold_input(np.zeros((1, 1, 10, 1)), 4)


@pytest.mark.parametrize("W_out", [12, 11, 9])
def test_unfold_inverts_fold_and_crops(oracle, W_out):
    F, Co, N, H = 4, 3, 2, 2
    y_full = rng(6).standard_normal((N, H, 12, Co))
    yf = oracle.fold_input(y_full, F)               # folded layout of a width-12 tensor
    y = oracle.unfold_output(yf, F, Co, W_out)
    assert y.shape == (N, H, W_out, Co)
    assert np.array_equal(y, y_full[:, :, :W_out, :])


# ----------------------------------------------------------------------------
# filter expansion
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("KH,C,Co,F", [(5, 1, 1, 8), (3, 1, 4, 4), (2, 3, 2, 8), (1, 2, 5, 3)])
def test_expand_kw1_is_kronecker_identity(oracle, KH, C, Co, F):
    """paper: Eq. filter_construct and the Kronecker-product remark."""
    w = rng(7).standard_normal((KH, 1, C, Co))
    we = oracle.expand_filter(w, F, 0)
    assert we.shape == (KH, 1, F * C, F * Co)
    for kh in range(KH):
        assert np.array_equal(we[kh, 0], np.kron(np.eye(F), w[kh, 0]))
    assert np.count_nonzero(we) == F * np.count_nonzero(w)


def test_expand_matches_listing_construction(oracle):
    """The appendix builds the filter by writing w into [:, :, f, f*Cout:(f+1)*Cout]."""
    K, F, Cout = 5, 8, 1
    w = rng(8).standard_normal((K, 1, 1, Cout))
    ref = np.zeros((K, 1, F, F * Cout))
    for f in range(F):
        ref[:, :, f, f * Cout:(f + 1) * Cout] = w[:, :, 0, :]
    assert np.array_equal(oracle.expand_filter(w, F, 0), ref)


def probe_expanded_filter(oracle, w, F, p_w, Wf_probe=5):
    """Brute force: recover the folded filter as the linear map it must be, by
    pushing one-hot *folded* inputs through the ORIGINAL direct convolution.
    Returns the [KH, KWf, F*C, F*Co] tensor read off at an interior column."""
    KH, KW, C, Co = w.shape
    sh = oracle.folded_shapes(F * Wf_probe, KW, p_w, F)
    d_min, KWf = sh["d_min"], sh["KWf"]
    W = F * Wf_probe
    ph = 0
    H = KH  # VALID along H -> a single output row; tap kh reads input row kh
    centre = Wf_probe // 2
    out = np.zeros((KH, KWf, F * C, F * Co))
    assert centre + d_min >= 0 and centre + sh["d_max"] < Wf_probe
    for kh in range(KH):
        for dd in range(KWf):
            for cp in range(F * C):
                xf = np.zeros((1, H, Wf_probe, F * C))
                xf[0, kh, centre + d_min + dd, cp] = 1.0
                x = xf.reshape(1, H, W, C)           # un-fold the probe (pure reshape)
                y = oracle.conv_direct(x, w, None, ph, p_w)
                # fold the output row and read the centre column
                W_out = y.shape[2]
                ypad = np.zeros((1, 1, sh["Wf_out"] * F, Co))
                ypad[:, :, :W_out] = y
                out[kh, dd, cp, :] = ypad.reshape(1, 1, sh["Wf_out"], F * Co)[0, 0, centre]
    return out


EXPAND_CASES = [
    # KH, KW, C, Co, F, p_w
    (3, 3, 3, 2, 4, 1),
    (1, 9, 1, 2, 8, 4),     # Conv1d, KW > F
    (2, 4, 2, 1, 4, 2),     # even kernel
    (3, 3, 1, 1, 2, 0),     # VALID
    (1, 5, 2, 2, 2, 2),     # KW > 2F
    (2, 3, 2, 3, 1, 1),     # F = 1
    (1, 3, 1, 2, 16, 1),
    (1, 2, 1, 1, 3, 3),     # pad beyond the kernel
]


@pytest.mark.parametrize("KH,KW,C,Co,F,p", EXPAND_CASES)
def test_expand_equals_probed_linear_map(oracle, KH, KW, C, Co, F, p):
    w = rng(9).standard_normal((KH, KW, C, Co))
    we = oracle.expand_filter(w, F, p)
    probed = probe_expanded_filter(oracle, w, F, p)
    assert we.shape == probed.shape
    assert np.array_equal(we, probed)


@pytest.mark.parametrize("KH,KW,C,Co,F,p", EXPAND_CASES)
def test_expand_block_structure(oracle, KH, KW, C, Co, F, p):
    w = rng(10).standard_normal((KH, KW, C, Co))  # almost surely no exact zeros
    we = oracle.expand_filter(w, F, p)
    KWf = we.shape[1]
    blocks = we.reshape(KH, KWf, F, C, F, Co)
    nz_blocks = np.any(blocks != 0, axis=(3, 5))          # [KH, KWf, F(f), F(g)]
    assert np.all(nz_blocks.sum(axis=(1, 2, 3)) == F * KW)   # F*KW blocks per kh
    assert np.count_nonzero(we) == F * w.size                 # every weight exactly F times
    assert np.all(nz_blocks.sum(axis=(1, 2)) == KW)           # each output slot g sees KW taps
    if F == 1:
        assert np.array_equal(we, w)


def brute_d_range(KW, p, F):
    ds = [(g + kw - p) // F for g in range(F) for kw in range(KW)]
    return min(ds), max(ds)


@pytest.mark.parametrize("W,KW,p,F", [(224, 3, 1, 16), (112, 3, 1, 4), (16000, 9, 4, 32), (32, 3, 1, 8),
                                       (64, 1, 0, 8), (12, 4, 2, 4), (12, 3, 0, 4), (10, 5, 2, 2), (9, 2, 3, 3)])
def test_folded_shapes_by_enumeration(oracle, W, KW, p, F):
    sh = oracle.folded_shapes(W, KW, p, F)
    dmin, dmax = brute_d_range(KW, p, F)
    assert (sh["d_min"], sh["d_max"], sh["KWf"]) == (dmin, dmax, dmax - dmin + 1)
    assert sh["Wf"] == W // F
    assert sh["W_out"] == W + 2 * p - KW + 1
    assert sh["Wf_out"] == -(-sh["W_out"] // F)
    # pads: every folded column any output slot can touch must exist after padding
    lo = min(wp + d for wp in range(sh["Wf_out"]) for d in (dmin, dmax))
    hi = max(wp + d for wp in range(sh["Wf_out"]) for d in (dmin, dmax))
    assert sh["pad_left_f"] == -lo
    assert sh["pad_right_f"] == hi - (sh["Wf"] - 1)


def test_same_padding_configs_have_three_folded_taps(oracle):
    for (W, KW, p, F) in [(32, 3, 1, 8), (224, 3, 1, 16), (112, 3, 1, 4), (16000, 9, 4, 32), (112, 3, 1, 16)]:
        sh = oracle.folded_shapes(W, KW, p, F)
        assert (sh["KWf"], sh["pad_left_f"], sh["pad_right_f"]) == (3, 1, 1)
        assert sh["Wf_out"] * F == sh["W_out"] == W


def test_tile_bias_is_tile(oracle):
    b = rng(11).standard_normal(5)
    assert np.array_equal(oracle.tile_bias(b, 4), np.tile(b, 4))


def test_pad_channels(oracle):
    x = rng(12).standard_normal((2, 3, 4, 3))
    xp = oracle.pad_channels(x, 8)
    assert xp.shape == (2, 3, 4, 8)
    assert np.array_equal(xp[..., :3], x) and np.all(xp[..., 3:] == 0)


# ----------------------------------------------------------------------------
# the rewrite as a whole
# ----------------------------------------------------------------------------
REWRITE_CASES = [
    # N, H, W, C, Co, KH, KW, ph, pw, F, bias
    (1, 32, 64, 1, 1, 5, 1, 0, 0, 8, True),     # the appendix listing
    (2, 6, 12, 1, 3, 3, 1, 0, 0, 4, True),      # proof setting: K x 1, C_in = 1
    (1, 8, 8, 3, 4, 3, 3, 1, 1, 4, False),      # same padding, taps along folded axis
    (2, 5, 16, 3, 2, 3, 3, 1, 1, 16, True),     # F == W
    (1, 1, 64, 1, 4, 1, 9, 0, 4, 32, False),    # Conv1d, KW < F
    (1, 1, 24, 1, 2, 1, 9, 0, 4, 4, True),      # KW > F
    (1, 6, 12, 2, 3, 3, 3, 0, 0, 4, True),      # VALID: ragged W_out = 10
    (1, 4, 12, 2, 2, 2, 4, 1, 2, 4, False),     # even kernel: W_out = 13 > W
    (1, 4, 12, 2, 2, 2, 4, 1, 1, 3, True),      # W_out = 11
    (2, 5, 7, 3, 3, 3, 3, 1, 1, 1, True),       # F = 1
    (1, 3, 6, 1, 1, 1, 2, 0, 3, 3, False),      # pad beyond kernel
    (1, 7, 8, 12, 5, 3, 3, 1, 1, 4, True),
]


@pytest.mark.parametrize("N,H,W,C,Co,KH,KW,ph,pw,F,hb", REWRITE_CASES)
def test_rewrite_equals_direct(oracle, N, H, W, C, Co, KH, KW, ph, pw, F, hb):
    """paper: section "Correctness of Width Folding Transformation" (Y' = Y)."""
    r = rng(20)
    x = r.standard_normal((N, H, W, C)); w = r.standard_normal((KH, KW, C, Co))
    b = r.standard_normal(Co) if hb else None
    yd = oracle.conv_direct(x, w, b, ph, pw)
    yr, parts = oracle.conv_rewrite(x, w, b, ph, pw, F, return_parts=True)
    assert yr.shape == yd.shape
    assert np.max(np.abs(yr - yd)) <= 1e-12
    sh = parts["shapes"]
    assert parts["xf"].shape == (N, H, W // F, F * C)
    assert parts["we"].shape == (KH, sh["KWf"], F * C, F * Co)
    assert parts["yf"].shape == (N, H + 2 * ph - KH + 1, sh["Wf_out"], F * Co)
    if F == 1:
        assert np.array_equal(yr, yd)      # identical arithmetic, identical bits
        assert np.array_equal(parts["we"], w)
    # torch as the outside opinion on the final result as well
    assert np.allclose(yr, torch_conv(x, w, b, ph, pw), rtol=0, atol=1e-12)


def test_rewrite_sweep_small(oracle):
    r = rng(21)
    count = 0
    for (KH, KW, p, F, C, Co) in itertools.product([1, 3], [1, 2, 3, 5], [0, 1, 2], [1, 2, 4], [1, 3], [1, 2]):
        W = 8
        H = 4
        ph = p if KH > 1 else 0
        if W + 2 * p - KW + 1 <= 0:
            continue
        x = r.standard_normal((1, H, W, C)); w = r.standard_normal((KH, KW, C, Co)); b = r.standard_normal(Co)
        yd = oracle.conv_direct(x, w, b, ph, p, relu=True)
        yr = oracle.conv_rewrite(x, w, b, ph, p, F, relu=True)
        assert yd.shape == yr.shape and np.max(np.abs(yd - yr)) <= 1e-12
        count += 1
    assert count > 100


def test_listing_shapes_and_tolerance(oracle):
    g = json.load(open(os.path.join(GOLD, "listing_shapes.json")))
    r = rng(22)
    x = r.standard_normal((g["B"], g["H"], g["W"], g["C_in"])).astype(np.float32)
    w = r.standard_normal((g["KH"], g["KW"], g["C_in"], g["C_out"])).astype(np.float32)
    b = r.standard_normal(g["C_out"]).astype(np.float32)
    y, parts = oracle.conv_rewrite(x, w, b, 0, 0, g["F"], return_parts=True)
    assert list(parts["xf"].shape) == g["x_folded_shape"]
    assert list(parts["we"].shape) == g["filter_expanded_shape"]
    assert list(parts["bf"].shape) == g["bias_expanded_shape"]
    assert list(parts["yf"].shape) == g["y_folded_shape"]
    assert list(y.shape[:3]) == g["y_reconstructed_shape"] and y.shape[3] == 1
    assert np.max(np.abs(y - oracle.conv_direct(x, w, b, 0, 0))) <= g["atol_fp32"]


def test_ir_closed_form_shapes(oracle):
    g = json.load(open(os.path.join(GOLD, "ir_shapes.json")))
    for c in g["cases"]:
        x = np.zeros((c["B"], c["H"], c["W"], c["C_in"]))
        w = np.zeros((c["KH"], c["KW"], c["C_in"], c["C_out"]))
        assert list(oracle.fold_input(x, c["F"]).shape) == c["x_folded_shape"]
        assert list(oracle.expand_filter(w, c["F"], 0).shape) == c["filter_expanded_shape"]
        assert list(oracle.tile_bias(np.zeros(c["C_out"]), c["F"]).shape) == c["bias_expanded_shape"]


def test_conv_stack_matches_torch(oracle):
    r = rng(23)
    chans = [3, 5, 4, 6]
    x = r.standard_normal((2, 6, 8, 3))
    ws = [r.standard_normal((3, 3, chans[i], chans[i + 1])) * 0.3 for i in range(3)]
    y = oracle.conv_stack(x, ws, 1)
    a = x
    for i, w in enumerate(ws):
        a = torch_conv(a, w, None, 1, 1, relu=(i < 2))
    assert np.allclose(y, a, rtol=0, atol=1e-12)


def test_axis_pad_convention(oracle):
    assert oracle.axis_pads(3, 3, 1) == (1, 1)
    assert oracle.axis_pads(1, 9, 4) == (0, 4)
    assert oracle.axis_pads(5, 1, 2) == (2, 0)
    assert oracle.axis_pads(1, 1, 3) == (0, 0)


def test_one_by_one_conv_is_matmul(oracle):
    """paper: "GEMM as a 1x1 Convolution" -- A[M,K] as x[1,1,M,K], B[K,N] as w[1,1,K,N]."""
    r = rng(30)
    A = r.standard_normal((24, 5)); B = r.standard_normal((5, 7))
    y = oracle.conv_direct(A.reshape(1, 1, 24, 5), B.reshape(1, 1, 5, 7), None, 0, 0)
    assert np.allclose(y.reshape(24, 7), A @ B, rtol=0, atol=1e-13)
    # folding rows of A into channels leaves the product unchanged; the expanded filter is I_F (x) B
    yr, parts = oracle.conv_rewrite(A.reshape(1, 1, 24, 5), B.reshape(1, 1, 5, 7), None, 0, 0, 4, return_parts=True)
    assert np.max(np.abs(yr.reshape(24, 7) - A @ B)) <= 1e-12
    assert np.array_equal(parts["we"][0, 0], np.kron(np.eye(4), B))
    # any H x W layout of the M rows gives the same product (a 1x1 kernel couples no two positions)
    y2 = oracle.conv_direct(A.reshape(1, 4, 6, 5), B.reshape(1, 1, 5, 7), None, 0, 0)
    assert np.array_equal(y2.reshape(24, 7), y.reshape(24, 7))
