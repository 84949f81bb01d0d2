"""libfoldconv: width-folded NHWC convolution for MI355X (gfx950).

Thin Python binding over the C ABI in ``include/foldconv.h``.  The shared
library is loaded on first use; importing the package loads nothing.
"""
from .binding import (  # noqa: F401
    FLAG_DENSE_K,
    FLAG_FILTER_COMPACT,
    FLAG_FILTER_PACKED,
    FLAG_KEEP_FOLDED,
    FLAG_RELU,
    FoldconvError,
    Plan,
    conv_padded_forward,
    foldconv_expand_filter,
    foldconv_fold_input,
    foldconv_forward,
    foldconv_pack_filter,
    foldconv_pack_filter_compact,
    foldconv_plan,
    foldconv_plan_gemm,
    foldconv_choose_fold,
    foldconv_plan_destroy,
    foldconv_plan_query,
    foldconv_strerror,
    foldconv_unfold_output,
    library_path,
    load_library,
)
