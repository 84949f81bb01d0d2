/*
 * libfoldconv -- width-folded NHWC convolution for gfx950 (MI355X).
 *
 * C ABI.  Every tensor pointer is a DEVICE pointer owned by the caller; the
 * library allocates no device memory, never frees anything the caller passed
 * and never synchronises: each call enqueues its kernels on `stream`
 * (a hipStream_t passed as void*, NULL = the default stream) and returns.
 * Inputs are read-only, outputs are fully overwritten.  Every function
 * returns FOLDCONV_OK (0) or a negative status; nothing throws across the
 * boundary.  A plan is host memory owned by the library until
 * foldconv_plan_destroy().
 *
 * Notation (paper: Algorithm 1, REQUIRE; section "Width-Folding
 * Transformation as an IR Transformation"):
 *   x  [N][H][W][C_in]            input, NHWC, row-major
 *   w  [KH][KW][C_in][C_out]      filter, HWIO
 *   b  [C_out]                    bias, same dtype as x
 *   F                             fold factor; W must be divisible by F
 *   x' [N][H][W/F][F*C_in]        folded input      (Eq. "width_fold_def")
 *   w' [KH][KW'][F*C_in][F*C_out] expanded filter   (Eq. "filter_construct")
 *   y' [N][H_out][W'_out][F*C_out] folded output    (Eq. "new_conv_H")
 *   y  [N][H_out][W_out][C_out]   reconstructed output ("Reconstruct" step)
 * Stride 1, cross-correlation (no kernel flip), symmetric zero padding `pad`
 * applied along an axis only when the kernel extends along it (KH > 1 for H,
 * KW > 1 for W), so Conv1d is H = KH = 1.
 *
 * The paper defines and proves the rewrite for a K x 1 kernel with C_in = 1
 * (convolution along H only).  For taps along the folded axis the expanded
 * filter becomes block-banded over KW' = d_max - d_min + 1 folded taps,
 *   d_min = floor(-p/F),  d_max = floor((F + KW - 2 - p)/F),
 *   w'[kh][d-d_min][f*C_in+c][g*C_out+co] = w[kh][F*d+f-g+p][c][co]
 * when that tap index lies in [0, KW), else 0; for KW = 1, p = 0 this is the
 * paper's block diagonal.
 */
#ifndef FOLDCONV_H
#define FOLDCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FOLDCONV_API __attribute__((visibility("default")))

typedef struct foldconv_plan_s *foldconv_plan_t;

typedef enum { FOLDCONV_F32 = 0, FOLDCONV_F16 = 1, FOLDCONV_BF16 = 2 } foldconv_dtype_t;

enum {
    FOLDCONV_OK = 0,
    FOLDCONV_ERR_BADARG = -1,      /* null pointer, non-positive size, unknown dtype/flag     */
    FOLDCONV_ERR_INDIVISIBLE = -2, /* W % F != 0 (paper: guard at the top of Algorithm 1)     */
    FOLDCONV_ERR_UNSUPPORTED = -3, /* empty output, sizes beyond 32-bit tile indexing         */
    FOLDCONV_ERR_WORKSPACE = -4,   /* workspace missing, too small, not 256-byte aligned, or
                                      claimed to hold a filter this plan never wrote there    */
    FOLDCONV_ERR_HIP = -5,         /* a HIP launch failed; hipGetLastError() was consumed     */
    FOLDCONV_ERR_SCRATCH = -6      /* the problem needs more than FOLDCONV_STATIC_SCRATCH_BYTES
                                      (foldconv_forward_static only)                          */
};

enum {
    FOLDCONV_FLAG_RELU = 1u,          /* y = max(0, conv + bias)                               */
    FOLDCONV_FLAG_DENSE_K = 2u,       /* walk every K-step of w', structural zeros included,
                                         instead of only the band that can be non-zero for the
                                         output slots of a tile.  Same result for finite data.
                                         (An fp32 plan given the compact filter walks the band
                                         where the dense walk would not fit the streaming kernel:
                                         the off-band blocks do not exist in that storage.)    */
    FOLDCONV_FLAG_KEEP_FOLDED = 4u,   /* write y' [N][H_out][W'_out][F*C_out], not y           */
    FOLDCONV_FLAG_FILTER_PACKED = 8u, /* workspace already holds the packed filter written by a
                                         previous call with the same plan and the same filter
                                         (weights are static after training): skip re-packing.
                                         The plan remembers the workspace it last packed into;
                                         any other pointer is FOLDCONV_ERR_WORKSPACE           */
    FOLDCONV_FLAG_FILTER_COMPACT = 16u, /* workspace holds the compact filter written by
                                         foldconv_pack_filter_compact (only the non-zero blocks
                                         of w'); w_exp is not read and may be NULL              */
    FOLDCONV_FLAG_OUT_NCHW = 32u,     /* write y channels-first, [N][C_out][H_out][W_out] of the
                                         image, in the same launch (no y' round trip through
                                         memory), for width- and height-folded plans.  Only where
                                         shapes.out_nchw_fused is 1, else
                                         FOLDCONV_ERR_UNSUPPORTED; excludes KEEP_FOLDED          */
    FOLDCONV_FLAG_UNPACED = 64u,      /* do not pace the store stream.  Long write-bound launches
                                         of the streaming kernels hold each wave's store burst to a
                                         schedule on the GPU's wall clock, set for a launch that
                                         has the whole memory system to itself (about 10 % faster
                                         than letting the waves overrun it).  A caller that runs
                                         other work beside the launch, or wants to measure the
                                         difference, passes this flag.  Same result either way.
                                         Also accepted by conv_padded_forward                    */
    FOLDCONV_FLAG_IN_NCHW = 128u      /* x_fold is the channels-first image itself,
                                         [N][C_in][H][W] (what foldconv_fold_input_nchw would
                                         read): the launch applies the fold in its load
                                         addressing and no folded copy is made.  Only together
                                         with FOLDCONV_FLAG_OUT_NCHW (FOLDCONV_ERR_BADARG
                                         without), where shapes.out_nchw_fused is 1; a width fold
                                         must also fit the input rows of a tile in LDS beside
                                         its output tiles (W a multiple of 8, H_out * W'_out a
                                         multiple of 32, W_out <= W, at most F*C_out 16-byte pieces
                                         in those rows); else FOLDCONV_ERR_UNSUPPORTED and the
                                         caller runs foldconv_fold_input_nchw first.  Same bits
                                         as the two-step route                                     */
};

/* Which image axis of a channels-first (NCHW) tensor is folded into the channels. */
enum { FOLDCONV_FOLD_W = 0, FOLDCONV_FOLD_H = 1 };

/* Everything a caller needs to size buffers and to report throughput. */
typedef struct foldconv_shapes_s {
    int32_t N, H, W, C_in, C_out, KH, KW, pad, F, dtype;
    int32_t pad_h, pad_w;           /* per-axis padding actually applied                     */
    int32_t W_fold;                 /* W / F                                                  */
    int32_t C_fold;                 /* F * C_in                                               */
    int32_t Co_fold;                /* F * C_out  (GEMM N)                                    */
    int32_t d_min, d_max, KW_fold;  /* folded tap range and count                             */
    int32_t pad_left_fold, pad_right_fold; /* zero columns the folded problem needs          */
    int32_t H_out, W_out, W_out_fold;      /* W_out_fold = ceil(W_out / F)                    */
    int32_t unfold_is_alias;        /* 1 when y and y' are the same bytes (W_out == F*W'_out) */
    int32_t C_pad;                  /* input channel count used by conv_padded_forward        */
    int32_t C_out_pad;              /* its output channel count (C_out rounded up to 8 for
                                       16-bit types; the result is cropped back to C_out)     */
    int32_t elem_bytes;
    int32_t conv_kernel;            /* 0 = gather MFMA, 1 = LDS-tiled MFMA, 2 = streaming MFMA
                                       (which kernel foldconv_forward will launch)            */
    int32_t padded_kernel;          /* same, for conv_padded_forward                          */
    int32_t fold_axis;              /* FOLDCONV_FOLD_W; FOLDCONV_FOLD_H for a plan made by
                                       foldconv_plan_nchw with height folding: then H, W, KH, KW
                                       and the *_out fields above describe the transposed image */
    int32_t out_nchw_fused;         /* 1 when foldconv_forward accepts FOLDCONV_FLAG_OUT_NCHW:
                                       16-bit plan on the streaming kernel, F*C_out a multiple of
                                       64 and at most 1024, C_out a multiple of 4, y below 4 GiB;
                                       width fold: F a multiple of 8 and W_out == F*W_out_fold;
                                       height fold: the image's W_out a multiple of 8, F even   */
    int32_t prefer_compact;         /* hint: 1 when foldconv_forward is expected to run faster from
                                       the compact filter than from packed w' (large-K layers whose
                                       packed band would crowd the input out of the L2: measured
                                       10-13 % on the 68 -> 132 and 132 -> 256 layers), else 0   */
    int64_t gemm_M, gemm_N, gemm_K; /* implicit GEMM of the folded problem, dense K           */
    int64_t x_bytes, w_bytes, bias_bytes, w_exp_bytes, y_bytes, y_fold_bytes;
    int64_t workspace_bytes;        /* for foldconv_forward / foldconv_pack_filter            */
    int64_t padded_workspace_bytes; /* for conv_padded_forward                                */
    int64_t filter_compact_bytes;   /* for foldconv_pack_filter_compact and foldconv_forward
                                       with FOLDCONV_FLAG_FILTER_COMPACT                      */
    double useful_flops;            /* 2*N*H_out*W_out*C_out*KH*KW*C_in                       */
    double issued_flops_dense;      /* MFMA flops issued with FOLDCONV_FLAG_DENSE_K           */
    double issued_flops_band;       /* MFMA flops issued by the default band walk             */
    double issued_flops_padded;     /* MFMA flops issued by conv_padded_forward               */
    double model_seconds;           /* the fold-factor cost model's estimate of one
                                       foldconv_forward (band walk, prepared filter); what
                                       foldconv_choose_fold compares across fold factors      */
} foldconv_shapes_t;

/*
 * Build a plan: legality test and all closed forms of the folded problem.
 * paper: Algorithm 1 (guard, shapes of X_f, W_f', b'); legality paragraph of
 * "Compiler-Level Realization in MLIR".  Unlike Algorithm 1 an illegal fold
 * is an error (FOLDCONV_ERR_INDIVISIBLE), not a silent fallback, and
 * C_in != 1 is supported through c' = f*C_in + c ("Mathematical
 * Perspective").  Host only; no GPU call is made.
 */
FOLDCONV_API int foldconv_plan(int N, int H, int W, int C_in, int C_out, int KH, int KW, int pad,
                  int fold_factor, foldconv_dtype_t dtype, foldconv_plan_t *out);

/*
 * Plan for a tall-skinny matrix product C[M][N] = A[M][K] * B[K][N] run as a
 * width-folded 1x1 convolution: A is the input x[1][1][M][K] (row-major A is
 * already that tensor), B is the filter w[1][1][K][N], C is y[1][1][M][N];
 * folding F rows of A into one pixel gives F*K aligned channels and the
 * expanded filter is the paper's block diagonal I_F (x) B.  M must be
 * divisible by F.  The returned plan is used with the same calls as any other
 * (expand, fold, forward, conv_padded_forward).
 * paper: section "Generalization to GEMM via 1x1 Convolution".
 */
FOLDCONV_API int foldconv_plan_gemm(long long M, int K, int N, int fold_factor, foldconv_dtype_t dtype,
                                    foldconv_plan_t *out);

/*
 * Plan for channels-first tensors  x [N][C_in][H][W],  w [C_out][C_in][KH][KW]
 * (OIHW),  y [N][C_out][H_out][W_out].  fold_axis = FOLDCONV_FOLD_H folds the
 * image height into the channels (H must be divisible by F), FOLDCONV_FOLD_W
 * the width.  Neither is an alias in this layout (no spatial axis is adjacent
 * to the channel axis), so the fold and the reconstruct are real re-indexing
 * kernels: foldconv_fold_input_nchw and foldconv_unfold_output_nchw, with
 * foldconv_expand_filter_oihw for the filter.  The folded tensors are kept
 * channels-last, x'[n][a][b'][f*C_in+c] with (a, F*b'+f) = (h, w) for
 * FOLD_W and (w, h) for FOLD_H, so foldconv_forward (with
 * FOLDCONV_FLAG_KEEP_FOLDED) and its kernels are the same as for NHWC; for
 * FOLD_H the plan is the width-fold plan of the transposed image and
 * shapes.{H,W,KH,KW,...} are reported in that transposed space.
 * paper: Introduction, "width folding for input in NHWC format (alternatively
 * height folding for NCHW format)".
 */
FOLDCONV_API int foldconv_plan_nchw(int N, int C_in, int H, int W, int C_out, int KH, int KW, int pad,
                                    int fold_factor, int fold_axis, foldconv_dtype_t dtype,
                                    foldconv_plan_t *out);

/*
 * Fold-factor choice: among the power-of-two factors F <= 64 that divide W,
 * the one with the smallest estimated time max(HBM bytes / sustained HBM rate,
 * issued MFMA flops / sustained MFMA rate), where a factor that leaves F*C_in
 * off the chunk alignment (a multiple of 4 elements; 8 for the full rate of
 * the 16-bit kernels) is charged the element-gather kernel's
 * rate; ties go to the smaller F.  *fold_factor receives the choice (1 = do not fold).
 * paper: "F is chosen to align with Tensor core tile sizes"; the "lightweight
 * cost model ... channel size, tensor core tile alignment, and arithmetic
 * intensity" of the MLIR section.  Host only.
 */
FOLDCONV_API int foldconv_choose_fold(int N, int H, int W, int C_in, int C_out, int KH, int KW, int pad,
                                      foldconv_dtype_t dtype, int *fold_factor);

/* Copy the plan's derived shapes into *out (host memory of the caller). */
FOLDCONV_API int foldconv_plan_query(foldconv_plan_t plan, foldconv_shapes_t *out);

/* Release a plan.  NULL is ignored. */
FOLDCONV_API void foldconv_plan_destroy(foldconv_plan_t plan);

/*
 * Structured filter expansion  w [KH][KW][C_in][C_out] -> w' (layout above),
 * zeros written explicitly; bit-exact copy of the filter values.
 * paper: Eq. "filter_construct"; Algorithm 1 "Define W_f' ... initialize to
 * zero" and the copy loop.  w_exp must hold shapes.w_exp_bytes.
 */
FOLDCONV_API int foldconv_expand_filter(foldconv_plan_t plan, const void *w, void *w_exp, void *stream);

/*
 * Input width fold  x -> x' with x'[n][h][w'][f*C_in+c] = x[n][h][F*w'+f][c].
 * paper: Eq. "width_fold_def"; Algorithm 1 loop nest.  In contiguous NHWC the
 * two tensors have identical linear offsets, so x_fold == x is legal and
 * returns at once without launching anything (the paper's listing folds with
 * a reshape); otherwise a vectorised copy of shapes.x_bytes is enqueued.
 * The buffers must not partially overlap.
 */
FOLDCONV_API int foldconv_fold_input(foldconv_plan_t plan, const void *x, void *x_fold, void *stream);

/*
 * Reconstruct  y'[n][h][w'][g*C_out+co] -> y[n][h][F*w'+g][co], dropping
 * columns F*w'+g >= W_out.  paper: "Let w = F w' + f" in the correctness
 * section; Reconstruct step of the IR formulation.  y == y_fold is legal only
 * when shapes.unfold_is_alias (then nothing is launched).
 */
FOLDCONV_API int foldconv_unfold_output(foldconv_plan_t plan, const void *y_fold, void *y, void *stream);

/*
 * Channels-first counterparts of the three data-movement steps.  All are
 * bit-exact moves; buffers must not overlap.
 *   foldconv_expand_filter_oihw: w [C_out][C_in][KH][KW] -> w' in the same
 *     canonical layout foldconv_expand_filter writes (Eq. "filter_construct"
 *     with the plan's folded axis in the role of W).
 *   foldconv_fold_input_nchw:  x [N][C_in][H][W] -> x' (shapes.x_bytes),
 *     x'[n][a][b'][f*C_in+c] = x[n][c][h][w] with (h, w) = (a, F*b'+f) for
 *     FOLD_W and (F*b'+f, a) for FOLD_H  (Eq. "width_fold_def" on that axis).
 *   foldconv_unfold_output_nchw:  y' [N][H_out][W'_out][F*C_out] as written by
 *     foldconv_forward with FOLDCONV_FLAG_KEEP_FOLDED (plan space; the same
 *     bytes as the default output when shapes.unfold_is_alias)
 *     -> y [N][C_out][H_out][W_out] of the image, dropping folded slots at or
 *     beyond the output extent (Reconstruct step).
 * A plan made by foldconv_plan is taken as FOLDCONV_FOLD_W.
 * Where shapes.out_nchw_fused is 1, foldconv_forward with
 * FOLDCONV_FLAG_OUT_NCHW writes the same bytes as foldconv_forward with
 * FOLDCONV_FLAG_KEEP_FOLDED followed by foldconv_unfold_output_nchw, without
 * the intermediate tensor.
 */
FOLDCONV_API int foldconv_expand_filter_oihw(foldconv_plan_t plan, const void *w_oihw, void *w_exp, void *stream);
FOLDCONV_API int foldconv_fold_input_nchw(foldconv_plan_t plan, const void *x_nchw, void *x_fold, void *stream);
FOLDCONV_API int foldconv_unfold_output_nchw(foldconv_plan_t plan, const void *y_fold, void *y_nchw, void *stream);

/*
 * Re-order w' into the operand order of the MFMA kernels (8 consecutive K
 * values of one output column per 16 bytes) inside `workspace`.  Optional:
 * foldconv_forward does this itself unless FOLDCONV_FLAG_FILTER_PACKED is
 * given.  Needs shapes.workspace_bytes (0 when the plan runs the gather
 * kernel, which reads w' directly; then this is a no-op).
 */
FOLDCONV_API int foldconv_pack_filter(foldconv_plan_t plan, const void *w_exp, void *workspace,
                         size_t workspace_bytes, void *stream);

/*
 * Compact storage of the expanded filter: only the non-zero blocks of w' are
 * kept.  Every output slot g uses the same KW*C_in x C_out tap matrix per kh,
 * placed (g-p)*C_in rows into the folded K window; the workspace receives one
 * zero-padded copy of that matrix per kh and per alignment of the placement
 * against the kernels' 8-row chunks (8/gcd(C_in,8) copies), built straight
 * from the ORIGINAL filter w [KH][KW][C_in][C_out] -- w' is never materialised.
 * Size: shapes.filter_compact_bytes (about KW/(KW'*F) of w').  Use the
 * workspace with foldconv_forward (same plan) and FOLDCONV_FLAG_FILTER_COMPACT;
 * results are bit-identical to the packed-w' route.
 * paper: section "Potential Optimizations for Sparsity and Quantization"
 * (store just the non-zero blocks of the block-structured filter).
 */
FOLDCONV_API int foldconv_pack_filter_compact(foldconv_plan_t plan, const void *w, void *workspace,
                                              size_t workspace_bytes, void *stream);

/*
 * Folded convolution + bias (+ReLU) + reconstruct:
 *   y'[n][h][w'][g*C_out+co] = b[co] + sum_{kh,d,c'} x'[n][h+kh-pad_h][w'+d][c'] * w'[kh][d-d_min][c'][g*C_out+co]
 * with out-of-range x' read as zero, fp32 accumulation, one rounding to the
 * plan dtype, written straight into y (reconstructed layout) unless
 * FOLDCONV_FLAG_KEEP_FOLDED.  paper: Eq. "new_conv_H"; Eq. "bias_construct"
 * (the replicated bias is read as b[n mod C_out]); Reconstruct step.
 * bias may be NULL.  workspace: shapes.workspace_bytes, 256-byte aligned,
 * may be NULL when that is 0; with FOLDCONV_FLAG_FILTER_COMPACT it is the
 * compact filter (shapes.filter_compact_bytes) and w_exp is ignored.
 * With FOLDCONV_FLAG_OUT_NCHW the reconstructed output is written
 * channels-first, y[n][co][h][F*w'+g] for a width fold and
 * y[n][co][F*h'+g][w] for a height fold (shapes.y_bytes, 16-byte aligned);
 * with FOLDCONV_FLAG_IN_NCHW as well, x_fold is the channels-first input
 * x[n][c][h][w] (paper: Eq. "width_fold_def", x'[n][h][w'][f*C+c] =
 * x[n][c][h][F*w'+f], resp. the same along h, applied on the fly).
 */
FOLDCONV_API int foldconv_forward(foldconv_plan_t plan, const void *x_fold, const void *w_exp,
                     const void *bias, void *y, void *workspace, size_t workspace_bytes,
                     unsigned flags, void *stream);

/*
 * foldconv_forward for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same result, same kernels and same arguments as
 * foldconv_forward, except that the kernel-order copy of w' is written to a
 * device array inside the library (FOLDCONV_STATIC_SCRATCH_BYTES per GPU the
 * library runs on, held until the process ends) instead of a caller
 * workspace.  Nothing is allocated or freed, here or in anything it calls.
 *   - plans with shapes.workspace_bytes above FOLDCONV_STATIC_SCRATCH_BYTES
 *     return FOLDCONV_ERR_SCRATCH and launch nothing;
 *   - every call re-packs w' (the scratch keeps whatever the last call on
 *     this GPU wrote, for any plan), so FOLDCONV_FLAG_FILTER_PACKED and
 *     FOLDCONV_FLAG_FILTER_COMPACT are FOLDCONV_ERR_BADARG here;
 *   - all calls on one GPU share the one array: calls whose kernels may
 *     overlap on that GPU (different streams, graphs replayed concurrently)
 *     race; calls on one stream are ordered and safe;
 *   - the first call on each GPU looks the array's device address up
 *     (hipGetSymbolAddress); make that call outside stream capture.
 */
#define FOLDCONV_STATIC_SCRATCH_BYTES (16u << 20)
FOLDCONV_API int foldconv_forward_static(foldconv_plan_t plan, const void *x_fold, const void *w_exp,
                                         const void *bias, void *y, unsigned flags, void *stream);

/*
 * Reference path: zero-pad C_in up to shapes.C_pad in the input and the
 * filter (and C_out up to shapes.C_out_pad in the filter and the bias), run
 * the same convolution kernels unfolded (F = 1), and crop the result back to
 * C_out channels when C_out was padded.
 * paper: the zero-padding alternative in the Introduction and in "Difference
 * from Channel Zero-Padding".  x and w are the ORIGINAL tensors; the padded
 * copies live in workspace (shapes.padded_workspace_bytes).  With
 * FOLDCONV_FLAG_FILTER_PACKED only the input is padded again (the workspace
 * must be the one this plan's previous call prepared).  Flags other than
 * FOLDCONV_FLAG_RELU, FOLDCONV_FLAG_FILTER_PACKED and FOLDCONV_FLAG_UNPACED
 * are FOLDCONV_ERR_BADARG: the reference path has no folded layout and no
 * structural zeros to walk.
 */
FOLDCONV_API int conv_padded_forward(foldconv_plan_t plan, const void *x, const void *w, const void *bias,
                        void *y, void *workspace, size_t workspace_bytes, unsigned flags,
                        void *stream);

/* Static text for a status code. */
FOLDCONV_API const char *foldconv_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* FOLDCONV_H */
