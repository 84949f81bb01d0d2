// The extern "C" entry points that enqueue GPU work: argument checks,
// workspace carving and the choice between the convolution kernels.
#include <stdint.h>

#include "geom.h"
#include "launch.h"

static bool plan_ok(foldconv_plan_t p) { return p && p->magic == FOLDCONV_MAGIC; }
static bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }
static int hip_status(int e) { return e == 0 ? FOLDCONV_OK : FOLDCONV_ERR_HIP; }

static const unsigned kAllFlags =
    FOLDCONV_FLAG_RELU | FOLDCONV_FLAG_DENSE_K | FOLDCONV_FLAG_KEEP_FOLDED | FOLDCONV_FLAG_FILTER_PACKED |
    FOLDCONV_FLAG_FILTER_COMPACT | FOLDCONV_FLAG_OUT_NCHW | FOLDCONV_FLAG_UNPACED | FOLDCONV_FLAG_IN_NCHW;

extern "C" int foldconv_expand_filter(foldconv_plan_t plan, const void *w, void *w_exp, void *stream) {
    if (!plan_ok(plan) || !w || !w_exp || w == w_exp) return FOLDCONV_ERR_BADARG;
    return hip_status(fc_launch_expand(plan, w, w_exp, 0, stream));
}

extern "C" int foldconv_expand_filter_oihw(foldconv_plan_t plan, const void *w_oihw, void *w_exp, void *stream) {
    if (!plan_ok(plan) || !w_oihw || !w_exp || w_oihw == w_exp) return FOLDCONV_ERR_BADARG;
    return hip_status(fc_launch_expand(plan, w_oihw, w_exp, 1, stream));
}

static bool overlap(const void *a, long long na, const void *b, long long nb) {
    const uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
    return x < y + (uintptr_t)nb && y < x + (uintptr_t)na;
}

extern "C" int foldconv_fold_input_nchw(foldconv_plan_t plan, const void *x_nchw, void *x_fold, void *stream) {
    if (!plan_ok(plan) || !x_nchw || !x_fold) return FOLDCONV_ERR_BADARG;
    const size_t eb = (size_t)plan->s.elem_bytes;
    if (!aligned(x_nchw, eb) || !aligned(x_fold, eb)) return FOLDCONV_ERR_BADARG;
    if (overlap(x_nchw, plan->s.x_bytes, x_fold, plan->s.x_bytes)) return FOLDCONV_ERR_BADARG;
    return hip_status(fc_launch_fold_nchw(plan, x_nchw, x_fold, stream));
}

extern "C" int foldconv_unfold_output_nchw(foldconv_plan_t plan, const void *y_fold, void *y_nchw, void *stream) {
    if (!plan_ok(plan) || !y_fold || !y_nchw) return FOLDCONV_ERR_BADARG;
    const size_t eb = (size_t)plan->s.elem_bytes;
    if (!aligned(y_fold, eb) || !aligned(y_nchw, eb)) return FOLDCONV_ERR_BADARG;
    if (overlap(y_fold, plan->s.y_fold_bytes, y_nchw, plan->s.y_bytes)) return FOLDCONV_ERR_BADARG;
    return hip_status(fc_launch_unfold_nchw(plan, y_fold, y_nchw, stream));
}

extern "C" int foldconv_fold_input(foldconv_plan_t plan, const void *x, void *x_fold, void *stream) {
    if (!plan_ok(plan) || !x || !x_fold) return FOLDCONV_ERR_BADARG;
    if (x == x_fold) return FOLDCONV_OK;  // identical linear offsets: the fold is the identity on bytes
    const uintptr_t a = (uintptr_t)x, b = (uintptr_t)x_fold, n = (uintptr_t)plan->s.x_bytes;
    if (a < b + n && b < a + n) return FOLDCONV_ERR_BADARG;  // partial overlap
    return hip_status(fc_launch_copy(x, x_fold, (size_t)plan->s.x_bytes, stream));
}

extern "C" int foldconv_unfold_output(foldconv_plan_t plan, const void *y_fold, void *y, void *stream) {
    if (!plan_ok(plan) || !y_fold || !y) return FOLDCONV_ERR_BADARG;
    if (y == y_fold) return plan->s.unfold_is_alias ? FOLDCONV_OK : FOLDCONV_ERR_BADARG;
    const uintptr_t a = (uintptr_t)y_fold, b = (uintptr_t)y;
    if (a < b + (uintptr_t)plan->s.y_bytes && b < a + (uintptr_t)plan->s.y_fold_bytes) return FOLDCONV_ERR_BADARG;
    if (plan->s.unfold_is_alias) return hip_status(fc_launch_copy(y_fold, y, (size_t)plan->s.y_bytes, stream));
    return hip_status(fc_launch_unfold(plan, y_fold, y, stream));
}

static int check_ws(const void *ws, size_t have, long long need) {
    if (need <= 0) return FOLDCONV_OK;
    if (!ws || have < (size_t)need || !aligned(ws, 256)) return FOLDCONV_ERR_WORKSPACE;
    return FOLDCONV_OK;
}

extern "C" int foldconv_pack_filter(foldconv_plan_t plan, const void *w_exp, void *workspace,
                                    size_t workspace_bytes, void *stream) {
    if (!plan_ok(plan) || !w_exp) return FOLDCONV_ERR_BADARG;
    if (plan->s.conv_kernel == FC_KERNEL_GATHER) return FOLDCONV_OK;
    int st = check_ws(workspace, workspace_bytes, plan->s.workspace_bytes);
    if (st) return st;
    if (!aligned(w_exp, (size_t)plan->s.elem_bytes)) return FOLDCONV_ERR_BADARG;
    st = hip_status(fc_launch_pack(plan->fold, plan->s.elem_bytes, w_exp, workspace, stream));
    if (st == FOLDCONV_OK) fc_stamp(&plan->packed_ws, workspace);
    return st;
}

extern "C" int foldconv_pack_filter_compact(foldconv_plan_t plan, const void *w, void *workspace,
                                            size_t workspace_bytes, void *stream) {
    if (!plan_ok(plan) || !w || w == workspace) return FOLDCONV_ERR_BADARG;
    int st = check_ws(workspace, workspace_bytes, plan->s.filter_compact_bytes);
    if (st) return st;
    if (!aligned(w, (size_t)plan->s.elem_bytes)) return FOLDCONV_ERR_BADARG;
    // The gather kernel indexes the original filter itself: its compact form is a copy of w.
    if (plan->s.conv_kernel == FC_KERNEL_GATHER)
        st = hip_status(fc_launch_copy(w, workspace, (size_t)plan->s.w_bytes, stream));
    else
        st = hip_status(fc_launch_compact(plan->fold, plan->s.elem_bytes, w, workspace, stream));
    if (st == FOLDCONV_OK) fc_stamp(&plan->compact_ws, workspace);
    return st;
}

extern "C" int foldconv_forward(foldconv_plan_t plan, const void *x_fold, const void *w_exp, const void *bias,
                                void *y, void *workspace, size_t workspace_bytes, unsigned flags, void *stream) {
    return fc_forward(plan, x_fold, w_exp, bias, y, workspace, workspace_bytes, flags, stream, true);
}

int fc_forward(foldconv_plan_t plan, const void *x_fold, const void *w_exp, const void *bias, void *y, void *workspace,
               size_t workspace_bytes, unsigned flags, void *stream, bool remember_workspace) {
    if (!plan_ok(plan) || !x_fold || !y) return FOLDCONV_ERR_BADARG;
    if (flags & ~kAllFlags) return FOLDCONV_ERR_BADARG;
    const bool compact = (flags & FOLDCONV_FLAG_FILTER_COMPACT) != 0;
    if (!compact && !w_exp) return FOLDCONV_ERR_BADARG;
    const foldconv_shapes_t &s = plan->s;
    const size_t eb = (size_t)s.elem_bytes;
    if (!aligned(x_fold, eb) || (!compact && !aligned(w_exp, eb)) || !aligned(y, eb) || (bias && !aligned(bias, eb)))
        return FOLDCONV_ERR_BADARG;
    ConvGeom g = plan->fold;
    g.relu = (flags & FOLDCONV_FLAG_RELU) ? 1 : 0;
    g.band = (flags & FOLDCONV_FLAG_DENSE_K) ? 0 : 1;
    g.has_bias = bias ? 1 : 0;
    g.unpaced = (flags & FOLDCONV_FLAG_UNPACED) ? 1 : 0;
    g.out_row = (flags & FOLDCONV_FLAG_KEEP_FOLDED) ? g.Wf_out * g.NCo : s.W_out * s.C_out;

    int kernel = s.conv_kernel;
    const bool out_nchw = (flags & FOLDCONV_FLAG_OUT_NCHW) != 0;
    const bool in_nchw = (flags & FOLDCONV_FLAG_IN_NCHW) != 0;
    if (in_nchw && !out_nchw) return FOLDCONV_ERR_BADARG;  // only the channels-first kernel gathers its input
    // (checked below, once the geometry of this call is known: a width fold must fit its stage of input rows in LDS)
    const bool hfold = plan->fold_axis == FOLDCONV_FOLD_H;
    if (out_nchw) {
        if (flags & FOLDCONV_FLAG_KEEP_FOLDED) return FOLDCONV_ERR_BADARG;
        g.out_row = s.W_out;
        int ks = 0;
        if (!s.out_nchw_fused || !fc_stream_nchw_ok(g, g.band, hfold, &ks)) return FOLDCONV_ERR_UNSUPPORTED;
        NchwStage stage;
        if (in_nchw && !hfold && !fc_stream_nchw_stage(g, &stage)) return FOLDCONV_ERR_UNSUPPORTED;
    }
    if (compact) {
        // every kernel takes its filter operand from the workspace
        int st = check_ws(workspace, workspace_bytes, s.filter_compact_bytes);
        if (st) return st;
        if (!fc_stamped(&plan->compact_ws, workspace)) return FOLDCONV_ERR_WORKSPACE;  // never packed by this plan
        if (kernel != FC_KERNEL_GATHER && (!aligned(x_fold, 16) || !aligned(y, 16))) return FOLDCONV_ERR_BADARG;
        g.compact = 1;
        if (kernel == FC_KERNEL_STREAM && !fc_tiled_ok(g)) {
            // Where the tiled kernel does not serve the layer (fp32, 8-byte operand chunks), a dense walk too long
            // for the streaming instances would run the element-gather kernel, which reads the canonical filter,
            // not this chunked form.  The off-band blocks do not exist in compact storage anyway: walk the band
            // (same result).
            StreamShape sh;
            if (!fc_stream_shape(g, g.band, &sh)) g.band = 1;
        }
        if (out_nchw)
            return hip_status(fc_launch_conv_stream_nchw((foldconv_dtype_t)s.dtype, g, hfold, in_nchw, x_fold, workspace, bias, y, stream));
        return hip_status(
            fc_launch_conv(kernel, (foldconv_dtype_t)s.dtype, g, x_fold, workspace, workspace, bias, y, stream));
    }
    if (kernel != FC_KERNEL_GATHER) {
        int st = check_ws(workspace, workspace_bytes, s.workspace_bytes);
        if (st) return st;
        // The vector kernels read 16-byte chunks; unaligned tensors are an error
        // rather than a silent change of kernel.
        if (!aligned(x_fold, 16) || !aligned(y, 16)) return FOLDCONV_ERR_BADARG;
        if (!(flags & FOLDCONV_FLAG_FILTER_PACKED)) {
            int e = fc_launch_pack(plan->fold, s.elem_bytes, w_exp, workspace, stream);
            if (e) return FOLDCONV_ERR_HIP;
            if (remember_workspace) fc_stamp(&plan->packed_ws, workspace);
        } else if (!fc_stamped(&plan->packed_ws, workspace)) {
            return FOLDCONV_ERR_WORKSPACE;  // never packed by this plan
        }
    }
    if (out_nchw)
        return hip_status(fc_launch_conv_stream_nchw((foldconv_dtype_t)s.dtype, g, hfold, in_nchw, x_fold, workspace, bias, y, stream));
    return hip_status(fc_launch_conv(kernel, (foldconv_dtype_t)s.dtype, g, x_fold, w_exp, workspace, bias, y, stream));
}

extern "C" int conv_padded_forward(foldconv_plan_t plan, const void *x, const void *w, const void *bias, void *y,
                                   void *workspace, size_t workspace_bytes, unsigned flags, void *stream) {
    if (!plan_ok(plan) || !x || !w || !y) return FOLDCONV_ERR_BADARG;
    // the reference path has one walk, one layout and one filter form
    if (flags & ~(unsigned)(FOLDCONV_FLAG_RELU | FOLDCONV_FLAG_FILTER_PACKED | FOLDCONV_FLAG_UNPACED)) return FOLDCONV_ERR_BADARG;
    const foldconv_shapes_t &s = plan->s;
    const size_t eb = (size_t)s.elem_bytes;
    if (!aligned(x, eb) || !aligned(w, eb) || !aligned(y, eb) || (bias && !aligned(bias, eb)))
        return FOLDCONV_ERR_BADARG;
    int st = check_ws(workspace, workspace_bytes, s.padded_workspace_bytes);
    if (st) return st;
    char *ws = (char *)workspace;
    void *x_pad = ws + plan->ws_xpad, *w_pad = ws + plan->ws_wpad, *w_pack = ws + plan->ws_wpack;
    const bool pad_out = s.C_out_pad != s.C_out;  // the kernels write C_out_pad channels per pixel, cropped below
    void *b_pad = ws + plan->ws_bpad, *y_pad = ws + plan->ws_ypad;
    const int kernel = s.padded_kernel;
    if (kernel != FC_KERNEL_GATHER && !pad_out && !aligned(y, 16)) return FOLDCONV_ERR_BADARG;

    if ((flags & FOLDCONV_FLAG_FILTER_PACKED) && !fc_stamped(&plan->padded_ws, workspace))
        return FOLDCONV_ERR_WORKSPACE;  // never prepared by this plan
    int e = fc_launch_pad_input(plan, x, x_pad, stream);
    if (e) return FOLDCONV_ERR_HIP;
    if (!(flags & FOLDCONV_FLAG_FILTER_PACKED)) {
        e = fc_launch_pad_filter(plan, w, w_pad, stream);
        if (e) return FOLDCONV_ERR_HIP;
        if (kernel != FC_KERNEL_GATHER) {
            e = fc_launch_pack(plan->padc, s.elem_bytes, w_pad, w_pack, stream);
            if (e) return FOLDCONV_ERR_HIP;
        }
        fc_stamp(&plan->padded_ws, workspace);
    }
    if (pad_out && bias) {  // the bias is an argument of every call: pad it every time
        e = fc_launch_pad_bias(plan, bias, b_pad, stream);
        if (e) return FOLDCONV_ERR_HIP;
    }
    ConvGeom g = plan->padc;
    g.relu = (flags & FOLDCONV_FLAG_RELU) ? 1 : 0;
    g.band = 1;
    g.has_bias = bias ? 1 : 0;
    g.unpaced = (flags & FOLDCONV_FLAG_UNPACED) ? 1 : 0;
    e = fc_launch_conv(kernel, (foldconv_dtype_t)s.dtype, g, x_pad, w_pad, w_pack, pad_out && bias ? b_pad : bias,
                       pad_out ? y_pad : y, stream);
    if (e) return FOLDCONV_ERR_HIP;
    if (pad_out) return hip_status(fc_launch_crop_channels(plan, y_pad, y, stream));
    return FOLDCONV_OK;
}
