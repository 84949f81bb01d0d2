"""ctypes binding of libfoldconv's C ABI (include/foldconv.h).

Argument marshalling only: tensors are torch CUDA tensors whose
``data_ptr()`` is handed to the library, the stream is torch's current HIP
stream.  No arithmetic happens here and there is no CPU fallback: if the
shared library is missing, loading raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfoldconv.so")

FLAG_RELU = 1
FLAG_DENSE_K = 2
FLAG_KEEP_FOLDED = 4
FLAG_FILTER_PACKED = 8
FLAG_FILTER_COMPACT = 16
FLAG_OUT_NCHW = 32
FLAG_UNPACED = 64
FLAG_IN_NCHW = 128
FOLD_W = 0
FOLD_H = 1
STATIC_SCRATCH_BYTES = 16 << 20

_DTYPE_CODE = {"float32": 0, "float16": 1, "bfloat16": 2}


class FoldconvError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (what, foldconv_strerror(status), status))


class Shapes(ctypes.Structure):
    """Mirror of foldconv_shapes_t."""

    _fields_ = (
        [(n, ctypes.c_int32) for n in (
            "N", "H", "W", "C_in", "C_out", "KH", "KW", "pad", "F", "dtype", "pad_h", "pad_w",
            "W_fold", "C_fold", "Co_fold", "d_min", "d_max", "KW_fold", "pad_left_fold", "pad_right_fold",
            "H_out", "W_out", "W_out_fold", "unfold_is_alias", "C_pad", "C_out_pad", "elem_bytes", "conv_kernel",
            "padded_kernel", "fold_axis", "out_nchw_fused", "prefer_compact")]
        + [(n, ctypes.c_int64) for n in (
            "gemm_M", "gemm_N", "gemm_K", "x_bytes", "w_bytes", "bias_bytes", "w_exp_bytes", "y_bytes",
            "y_fold_bytes", "workspace_bytes", "padded_workspace_bytes", "filter_compact_bytes")]
        + [(n, ctypes.c_double) for n in (
            "useful_flops", "issued_flops_dense", "issued_flops_band", "issued_flops_padded", "model_seconds")]
    )

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


_lib = None


def library_path():
    return _LIB_PATH


def load_library():
    """Load libfoldconv.so (built in-tree by ``paper_2601_11608_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            "libfoldconv.so is not built: run `python -m paper_2601_11608_amd.build` "
            "(there is no fallback path)")
    try:
        import torch  # noqa: F401  -- loads the HIP runtime this process will share with the library
    except ImportError:
        pass
    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz, ui, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint, ctypes.c_int
    lib.foldconv_plan.argtypes = [ci] * 10 + [ctypes.POINTER(vp)]
    lib.foldconv_plan.restype = ci
    lib.foldconv_plan_nchw.argtypes = [ci] * 11 + [ctypes.POINTER(vp)]
    lib.foldconv_plan_nchw.restype = ci
    for name in ("foldconv_expand_filter_oihw", "foldconv_fold_input_nchw", "foldconv_unfold_output_nchw"):
        getattr(lib, name).argtypes = [vp, vp, vp, vp]
        getattr(lib, name).restype = ci
    lib.foldconv_plan_gemm.argtypes = [ctypes.c_longlong, ci, ci, ci, ci, ctypes.POINTER(vp)]
    lib.foldconv_plan_gemm.restype = ci
    lib.foldconv_choose_fold.argtypes = [ci] * 9 + [ctypes.POINTER(ci)]
    lib.foldconv_choose_fold.restype = ci
    lib.foldconv_plan_query.argtypes = [vp, ctypes.POINTER(Shapes)]
    lib.foldconv_plan_query.restype = ci
    lib.foldconv_plan_destroy.argtypes = [vp]
    lib.foldconv_plan_destroy.restype = None
    lib.foldconv_expand_filter.argtypes = [vp, vp, vp, vp]
    lib.foldconv_expand_filter.restype = ci
    lib.foldconv_fold_input.argtypes = [vp, vp, vp, vp]
    lib.foldconv_fold_input.restype = ci
    lib.foldconv_unfold_output.argtypes = [vp, vp, vp, vp]
    lib.foldconv_unfold_output.restype = ci
    lib.foldconv_pack_filter.argtypes = [vp, vp, vp, sz, vp]
    lib.foldconv_pack_filter.restype = ci
    lib.foldconv_pack_filter_compact.argtypes = [vp, vp, vp, sz, vp]
    lib.foldconv_pack_filter_compact.restype = ci
    lib.foldconv_forward.argtypes = [vp, vp, vp, vp, vp, vp, sz, ui, vp]
    lib.foldconv_forward.restype = ci
    lib.foldconv_forward_static.argtypes = [vp, vp, vp, vp, vp, ui, vp]
    lib.foldconv_forward_static.restype = ci
    lib.conv_padded_forward.argtypes = [vp, vp, vp, vp, vp, vp, sz, ui, vp]
    lib.conv_padded_forward.restype = ci
    lib.foldconv_strerror.argtypes = [ci]
    lib.foldconv_strerror.restype = ctypes.c_char_p
    _lib = lib
    return lib


def foldconv_strerror(status):
    return load_library().foldconv_strerror(int(status)).decode()


class Plan:
    """Owns a foldconv_plan_t; ``.shapes`` is the queried foldconv_shapes_t."""

    def __init__(self, handle, shapes):
        self.handle = handle
        self.shapes = shapes

    def destroy(self):
        if self.handle:
            load_library().foldconv_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _check(status, what):
    if status != 0:
        raise FoldconvError(status, what)


def _dtype_code(dtype):
    if isinstance(dtype, int):
        return dtype
    name = str(dtype).replace("torch.", "")
    return _DTYPE_CODE[name]


def foldconv_plan(N, H, W, C_in, C_out, KH, KW, pad, fold_factor, dtype):
    lib = load_library()
    h = ctypes.c_void_p()
    _check(lib.foldconv_plan(N, H, W, C_in, C_out, KH, KW, pad, fold_factor, _dtype_code(dtype), ctypes.byref(h)),
           "foldconv_plan")
    plan = Plan(h, None)
    plan.shapes = foldconv_plan_query(plan)
    return plan


def foldconv_plan_nchw(N, C_in, H, W, C_out, KH, KW, pad, fold_factor, fold_axis, dtype):
    lib = load_library()
    h = ctypes.c_void_p()
    _check(lib.foldconv_plan_nchw(N, C_in, H, W, C_out, KH, KW, pad, fold_factor, fold_axis, _dtype_code(dtype),
                                  ctypes.byref(h)), "foldconv_plan_nchw")
    plan = Plan(h, None)
    plan.shapes = foldconv_plan_query(plan)
    return plan


def foldconv_plan_gemm(M, K, N, fold_factor, dtype):
    lib = load_library()
    h = ctypes.c_void_p()
    _check(lib.foldconv_plan_gemm(M, K, N, fold_factor, _dtype_code(dtype), ctypes.byref(h)), "foldconv_plan_gemm")
    plan = Plan(h, None)
    plan.shapes = foldconv_plan_query(plan)
    return plan


def foldconv_choose_fold(N, H, W, C_in, C_out, KH, KW, pad, dtype):
    f = ctypes.c_int(1)
    _check(load_library().foldconv_choose_fold(N, H, W, C_in, C_out, KH, KW, pad, _dtype_code(dtype),
                                               ctypes.byref(f)), "foldconv_choose_fold")
    return f.value


def foldconv_plan_query(plan):
    s = Shapes()
    _check(load_library().foldconv_plan_query(plan.handle, ctypes.byref(s)), "foldconv_plan_query")
    return s


def foldconv_plan_destroy(plan):
    plan.destroy()


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    if not t.is_cuda:
        raise ValueError("libfoldconv takes device tensors")
    if not t.is_contiguous():
        raise ValueError("libfoldconv takes contiguous tensors")
    return ctypes.c_void_p(t.data_ptr())


def _nbytes(t):
    return 0 if t is None else (t if isinstance(t, int) else t.numel() * t.element_size())


def _stream(stream):
    if stream is not None:
        return ctypes.c_void_p(stream if isinstance(stream, int) else stream.cuda_stream)
    import torch

    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _need(t, nbytes, name):
    if not isinstance(t, int) and t is not None and _nbytes(t) < nbytes:
        raise ValueError("%s holds %d bytes, needs %d" % (name, _nbytes(t), nbytes))


def foldconv_expand_filter(plan, w, w_exp, stream=None):
    s = plan.shapes
    _need(w, s.w_bytes, "w")
    _need(w_exp, s.w_exp_bytes, "w_exp")
    _check(load_library().foldconv_expand_filter(plan.handle, _ptr(w), _ptr(w_exp), _stream(stream)),
           "foldconv_expand_filter")


def foldconv_expand_filter_oihw(plan, w_oihw, w_exp, stream=None):
    s = plan.shapes
    _need(w_oihw, s.w_bytes, "w_oihw")
    _need(w_exp, s.w_exp_bytes, "w_exp")
    _check(load_library().foldconv_expand_filter_oihw(plan.handle, _ptr(w_oihw), _ptr(w_exp), _stream(stream)),
           "foldconv_expand_filter_oihw")


def foldconv_fold_input_nchw(plan, x_nchw, x_fold, stream=None):
    s = plan.shapes
    _need(x_nchw, s.x_bytes, "x_nchw")
    _need(x_fold, s.x_bytes, "x_fold")
    _check(load_library().foldconv_fold_input_nchw(plan.handle, _ptr(x_nchw), _ptr(x_fold), _stream(stream)),
           "foldconv_fold_input_nchw")


def foldconv_unfold_output_nchw(plan, y_fold, y_nchw, stream=None):
    s = plan.shapes
    _need(y_fold, s.y_fold_bytes, "y_fold")
    _need(y_nchw, s.y_bytes, "y_nchw")
    _check(load_library().foldconv_unfold_output_nchw(plan.handle, _ptr(y_fold), _ptr(y_nchw), _stream(stream)),
           "foldconv_unfold_output_nchw")


def foldconv_fold_input(plan, x, x_fold, stream=None):
    s = plan.shapes
    _need(x, s.x_bytes, "x")
    _need(x_fold, s.x_bytes, "x_fold")
    _check(load_library().foldconv_fold_input(plan.handle, _ptr(x), _ptr(x_fold), _stream(stream)),
           "foldconv_fold_input")


def foldconv_unfold_output(plan, y_fold, y, stream=None):
    s = plan.shapes
    _need(y_fold, s.y_fold_bytes, "y_fold")
    _need(y, s.y_bytes, "y")
    _check(load_library().foldconv_unfold_output(plan.handle, _ptr(y_fold), _ptr(y), _stream(stream)),
           "foldconv_unfold_output")


def foldconv_pack_filter(plan, w_exp, workspace, stream=None):
    s = plan.shapes
    _need(w_exp, s.w_exp_bytes, "w_exp")
    _check(load_library().foldconv_pack_filter(plan.handle, _ptr(w_exp), _ptr(workspace), _nbytes(workspace),
                                               _stream(stream)), "foldconv_pack_filter")


def foldconv_pack_filter_compact(plan, w, workspace, stream=None):
    s = plan.shapes
    _need(w, s.w_bytes, "w")
    _check(load_library().foldconv_pack_filter_compact(plan.handle, _ptr(w), _ptr(workspace), _nbytes(workspace),
                                                       _stream(stream)), "foldconv_pack_filter_compact")


def foldconv_forward(plan, x_fold, w_exp, bias, y, workspace=None, flags=0, stream=None):
    s = plan.shapes
    _need(x_fold, s.x_bytes, "x_fold")
    if not (flags & FLAG_FILTER_COMPACT):
        _need(w_exp, s.w_exp_bytes, "w_exp")
    _need(bias, s.bias_bytes, "bias")
    _need(y, s.y_fold_bytes if (flags & FLAG_KEEP_FOLDED) else s.y_bytes, "y")
    _check(load_library().foldconv_forward(plan.handle, _ptr(x_fold), _ptr(w_exp), _ptr(bias), _ptr(y),
                                           _ptr(workspace), _nbytes(workspace), flags, _stream(stream)),
           "foldconv_forward")


def foldconv_forward_static(plan, x_fold, w_exp, bias, y, flags=0, stream=None):
    s = plan.shapes
    _need(x_fold, s.x_bytes, "x_fold")
    _need(w_exp, s.w_exp_bytes, "w_exp")
    _need(bias, s.bias_bytes, "bias")
    _need(y, s.y_fold_bytes if (flags & FLAG_KEEP_FOLDED) else s.y_bytes, "y")
    _check(load_library().foldconv_forward_static(plan.handle, _ptr(x_fold), _ptr(w_exp), _ptr(bias), _ptr(y),
                                                  flags, _stream(stream)), "foldconv_forward_static")


def conv_padded_forward(plan, x, w, bias, y, workspace, flags=0, stream=None):
    s = plan.shapes
    _need(x, s.x_bytes, "x")
    _need(w, s.w_bytes, "w")
    _need(bias, s.bias_bytes, "bias")
    _need(y, s.y_bytes, "y")
    _check(load_library().conv_padded_forward(plan.handle, _ptr(x), _ptr(w), _ptr(bias), _ptr(y), _ptr(workspace),
                                              _nbytes(workspace), flags, _stream(stream)), "conv_padded_forward")
