"""TEST INFRASTRUCTURE ONLY: ctypes front end of the fp64 CPU oracle.

Everything here runs on the host in float64 through ``foldconv_oracle.c``.
The product (the HIP library and its binding) never imports this module;
only ``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg do.
This module imports nothing from the GPU package.

Array conventions: NHWC inputs ``x[N,H,W,C]``, HWIO filters
``w[KH,KW,C,Co]`` (paper: Algorithm 1, REQUIRE), numpy float64, C-contiguous.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "foldconv_oracle.c")
_LIB = os.path.join(_HERE, "libfoldconv_oracle.so")

_D = ctypes.POINTER(ctypes.c_double)
_I = ctypes.c_int


def build(force=False):
    """Compile the C oracle with gcc (-O2 -fopenmp).  Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", tmp, _SRC]
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_conv2d_nhwc.argtypes = [_D, _D, _D, _D] + [_I] * 12
        lib.oracle_conv2d_nhwc.restype = None
        lib.oracle_fold_input.argtypes = [_D, _D] + [_I] * 5
        lib.oracle_fold_input.restype = None
        lib.oracle_folded_shapes.argtypes = [_I, _I, _I, _I, ctypes.POINTER(_I)]
        lib.oracle_folded_shapes.restype = None
        lib.oracle_expand_filter.argtypes = [_D, _D] + [_I] * 6
        lib.oracle_expand_filter.restype = None
        lib.oracle_tile_bias.argtypes = [_D, _D, _I, _I]
        lib.oracle_tile_bias.restype = None
        lib.oracle_unfold_output.argtypes = [_D, _D] + [_I] * 6
        lib.oracle_unfold_output.restype = None
        lib.oracle_pad_channels.argtypes = [_D, _D, ctypes.c_size_t, _I, _I]
        lib.oracle_pad_channels.restype = None
        lib.oracle_conv2d_nchw.argtypes = [_D, _D, _D, _D] + [_I] * 12
        lib.oracle_conv2d_nchw.restype = None
        lib.oracle_fold_input_h_nchw.argtypes = [_D, _D] + [_I] * 5
        lib.oracle_fold_input_h_nchw.restype = None
        lib.oracle_expand_filter_h_oihw.argtypes = [_D, _D] + [_I] * 6
        lib.oracle_expand_filter_h_oihw.restype = None
        lib.oracle_unfold_output_h_nchw.argtypes = [_D, _D] + [_I] * 6
        lib.oracle_unfold_output_h_nchw.restype = None
        _lib = lib
    return _lib


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _p(a):
    return a.ctypes.data_as(_D)


def axis_pads(KH, KW, pad):
    """Padding convention of the C ABI: the single ``pad`` applies along an
    axis only if the kernel extends along it (Conv1d is H = KH = 1, padded
    along W only; a K x 1 kernel as in the paper's proof pads H only)."""
    return (pad if KH > 1 else 0), (pad if KW > 1 else 0)


def conv2d_general(x, w, b, pad_top, pad_left, H_out, W_out, relu=False):
    """Direct cross-correlation with explicit top/left pads and output extent."""
    x, w = _f64(x), _f64(w)
    N, H, W, C = x.shape
    KH, KW, C2, Co = w.shape
    assert C2 == C
    bb = None if b is None else _f64(b)
    y = np.empty((N, H_out, W_out, Co), dtype=np.float64)
    _load().oracle_conv2d_nhwc(
        _p(x), _p(w), None if bb is None else _p(bb), _p(y),
        N, H, W, C, Co, KH, KW, pad_top, pad_left, H_out, W_out, int(bool(relu)),
    )
    return y


def conv_direct(x, w, b=None, pad_h=0, pad_w=0, relu=False):
    """The definition: stride-1 cross-correlation with symmetric zero padding.
    paper: standard contraction in "Width Folding: Mathematical Perspective"."""
    N, H, W, C = x.shape
    KH, KW = w.shape[0], w.shape[1]
    H_out = H + 2 * pad_h - KH + 1
    W_out = W + 2 * pad_w - KW + 1
    return conv2d_general(x, w, b, pad_h, pad_w, H_out, W_out, relu)


def folded_shapes(W, KW, p, F):
    out = (_I * 8)()
    _load().oracle_folded_shapes(W, KW, p, F, out)
    keys = ["Wf", "d_min", "d_max", "KWf", "W_out", "Wf_out", "pad_left_f", "pad_right_f"]
    return dict(zip(keys, [int(v) for v in out]))


def fold_input(x, F):
    """paper: Eq. "width_fold_def" / the c' = f*C_in + c form."""
    x = _f64(x)
    N, H, W, C = x.shape
    assert W % F == 0, "Algorithm 1 guard: W mod F != 0"
    xf = np.empty((N, H, W // F, F * C), dtype=np.float64)
    _load().oracle_fold_input(_p(x), _p(xf), N, H, W, C, F)
    return xf


def expand_filter(w, F, p):
    """paper: Eq. "filter_construct", Algorithm 1.  ``p`` = width padding."""
    w = _f64(w)
    KH, KW, C, Co = w.shape
    sh = folded_shapes(F, KW, p, F)
    we = np.empty((KH, sh["KWf"], F * C, F * Co), dtype=np.float64)
    _load().oracle_expand_filter(_p(w), _p(we), KH, KW, C, Co, F, p)
    return we


def tile_bias(b, F):
    """paper: Eq. "bias_construct"."""
    b = _f64(b)
    bf = np.empty((F * b.shape[0],), dtype=np.float64)
    _load().oracle_tile_bias(_p(b), _p(bf), b.shape[0], F)
    return bf


def unfold_output(yf, F, Co, W_out):
    """paper: Reconstruct step (w = F w' + f)."""
    yf = _f64(yf)
    N, H_out, Wf_out, FCo = yf.shape
    assert FCo == F * Co
    y = np.empty((N, H_out, W_out, Co), dtype=np.float64)
    _load().oracle_unfold_output(_p(yf), _p(y), N, H_out, Wf_out, F, Co, W_out)
    return y


def pad_channels(x, C_pad):
    x = _f64(x)
    C = x.shape[-1]
    xp = np.empty(x.shape[:-1] + (C_pad,), dtype=np.float64)
    _load().oracle_pad_channels(_p(x), _p(xp), x.size // C, C, C_pad)
    return xp


def conv_rewrite(x, w, b=None, pad_h=0, pad_w=0, F=1, relu=False, return_parts=False):
    """The paper's rewrite on the CPU: fold -> expand -> replicate bias ->
    ordinary convolution on the folded shapes -> reconstruct.
    paper: Algorithm 1 followed by Eq. "new_conv_H" and the Reconstruct step.
    Used to validate the method itself against ``conv_direct``."""
    N, H, W, C = x.shape
    KH, KW, _, Co = w.shape
    sh = folded_shapes(W, KW, pad_w, F)
    xf = fold_input(x, F)
    we = expand_filter(w, F, pad_w)
    bf = None if b is None else tile_bias(b, F)
    H_out = H + 2 * pad_h - KH + 1
    yf = conv2d_general(xf, we, bf, pad_h, sh["pad_left_f"], H_out, sh["Wf_out"], relu)
    y = unfold_output(yf, F, Co, sh["W_out"])
    if return_parts:
        return y, dict(xf=xf, we=we, bf=bf, yf=yf, shapes=sh)
    return y


def conv_stack(x, ws, pad, relu_between=True):
    """Chain of stride-1 'same' convolutions with ReLU between layers, all in
    fp64 (no intermediate rounding)."""
    a = _f64(x)
    for i, w in enumerate(ws):
        ph, pw = axis_pads(w.shape[0], w.shape[1], pad)
        a = conv_direct(a, w, None, ph, pw, relu=(relu_between and i + 1 < len(ws)))
    return a


# --- channels-first tensors and height folding ---------------------------------
# paper: Introduction, "width folding for input in NHWC format (alternatively
# height folding for NCHW format)".  x[N,C,H,W], w[Co,C,KH,KW] (OIHW).

def conv2d_general_nchw(x, w, b, pad_top, pad_left, H_out, W_out, relu=False):
    x, w = _f64(x), _f64(w)
    N, C, H, W = x.shape
    Co, C2, KH, KW = w.shape
    assert C2 == C
    bb = None if b is None else _f64(b)
    y = np.empty((N, Co, H_out, W_out), dtype=np.float64)
    _load().oracle_conv2d_nchw(
        _p(x), _p(w), None if bb is None else _p(bb), _p(y),
        N, C, H, W, Co, KH, KW, pad_top, pad_left, H_out, W_out, int(bool(relu)),
    )
    return y


def conv_direct_nchw(x, w, b=None, pad_h=0, pad_w=0, relu=False):
    """The definition on channels-first tensors (stride 1, symmetric zero padding)."""
    N, C, H, W = x.shape
    KH, KW = w.shape[2], w.shape[3]
    return conv2d_general_nchw(x, w, b, pad_h, pad_w, H + 2 * pad_h - KH + 1, W + 2 * pad_w - KW + 1, relu)


def fold_input_h_nchw(x, F):
    """xh[n, f*C+c, h', w] = x[n, c, F*h'+f, w]."""
    x = _f64(x)
    N, C, H, W = x.shape
    assert H % F == 0, "guard: H mod F != 0"
    xh = np.empty((N, F * C, H // F, W), dtype=np.float64)
    _load().oracle_fold_input_h_nchw(_p(x), _p(xh), N, C, H, W, F)
    return xh


def expand_filter_h_oihw(w, F, p):
    """wh[g*Co+co, f*C+c, d-d_min, kw] = w[co, c, F*d+f-g+p, kw] (zero outside the tap range)."""
    w = _f64(w)
    Co, C, KH, KW = w.shape
    sh = folded_shapes(F, KH, p, F)
    wh = np.empty((F * Co, F * C, sh["KWf"], KW), dtype=np.float64)
    _load().oracle_expand_filter_h_oihw(_p(w), _p(wh), Co, C, KH, KW, F, p)
    return wh


def unfold_output_h_nchw(yh, F, Co, H_out):
    """y[n, co, F*h'+g, w] = yh[n, g*Co+co, h', w] for F*h'+g < H_out."""
    yh = _f64(yh)
    N, FCo, Hf_out, W_out = yh.shape
    assert FCo == F * Co
    y = np.empty((N, Co, H_out, W_out), dtype=np.float64)
    _load().oracle_unfold_output_h_nchw(_p(yh), _p(y), N, Co, Hf_out, W_out, F, H_out)
    return y


def conv_rewrite_h_nchw(x, w, b=None, pad_h=0, pad_w=0, F=1, relu=False, return_parts=False):
    """Height-folding rewrite on the CPU: fold H into channels, expand the filter along KH,
    replicate the bias, ordinary channels-first convolution on the folded shapes, reconstruct."""
    N, C, H, W = x.shape
    Co, _, KH, KW = w.shape
    sh = folded_shapes(H, KH, pad_h, F)          # the closed forms with H, KH in place of W, KW
    xh = fold_input_h_nchw(x, F)
    wh = expand_filter_h_oihw(w, F, pad_h)
    bf = None if b is None else tile_bias(b, F)
    W_out = W + 2 * pad_w - KW + 1
    yh = conv2d_general_nchw(xh, wh, bf, sh["pad_left_f"], pad_w, sh["Wf_out"], W_out, relu)
    y = unfold_output_h_nchw(yh, F, Co, sh["W_out"])
    if return_parts:
        return y, dict(xh=xh, wh=wh, bf=bf, yh=yh, shapes=sh)
    return y
