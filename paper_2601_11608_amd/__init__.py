"""libfoldconv: width-folded NHWC convolution for MI355X (gfx950).

Thin Python binding over the C ABI in ``include/foldconv.h``.  The shared
library is loaded on first use; importing the package loads nothing.
"""
from .binding import (  # noqa: F401
    FLAG_DENSE_K,
    FLAG_FILTER_COMPACT,
    FLAG_OUT_NCHW,
    FLAG_FILTER_PACKED,
    FLAG_KEEP_FOLDED,
    FLAG_RELU,
    FLAG_UNPACED,
    FOLD_H,
    FOLD_W,
    STATIC_SCRATCH_BYTES,
    FoldconvError,
    Plan,
    conv_padded_forward,
    foldconv_expand_filter,
    foldconv_expand_filter_oihw,
    foldconv_fold_input,
    foldconv_fold_input_nchw,
    foldconv_forward,
    foldconv_forward_static,
    foldconv_pack_filter,
    foldconv_pack_filter_compact,
    foldconv_plan,
    foldconv_plan_gemm,
    foldconv_plan_nchw,
    foldconv_choose_fold,
    foldconv_plan_destroy,
    foldconv_plan_query,
    foldconv_strerror,
    foldconv_unfold_output,
    foldconv_unfold_output_nchw,
    library_path,
    load_library,
)
