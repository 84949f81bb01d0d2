// Host-only part of libfoldconv: legality, closed forms of the folded
// problem, workspace layout, kernel choice and FLOP accounting.
// paper: Algorithm 1 (guard and the shapes of X_f, W_f', b'); the shapes in
// "Width-Folding Transformation as an IR Transformation"; legality paragraph
// of "Compiler-Level Realization in MLIR".
#include <limits.h>
#include <new>
#include <string.h>

#include "geom.h"
#include "launch.h"

static long long floor_div_ll(long long a, long long b) {
    long long q = a / b;
    if ((a % b) != 0 && ((a < 0) != (b < 0))) --q;
    return q;
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// MFMA flops issued by a kernel whose band window is taken per `tile_n`
// output columns, in K-steps of `kstep` elements aligned to `align`.  The
// LDS-tiled kernel walks K in blocks of 32 and multiplies whole tiles, the
// columns past F*C_out included (full_tiles).  bias_k: K extent of the extra
// rank-1 MFMA through which the vector kernels add the bias and initialise
// their accumulators (one 16-wide step per 32 x 32 tile, issued whether or
// not a bias is given; 0 for kernels that add the bias in fp32).
static double issued_flops(ConvGeom g, int band, int tile_n, int kstep, int align, bool full_tiles, int bias_k) {
    if (full_tiles) kstep = 32;
    g.band = band;
    double total = 0.0;
    for (int n0 = 0; n0 < g.NCo; n0 += tile_n) {
        int n1 = n0 + tile_n < g.NCo ? n0 + tile_n : g.NCo;
        int e_lo, e_hi;
        fc_band_window(g, n0, n1, align, &e_lo, &e_hi);
        long long steps = ((long long)(e_hi - e_lo) + kstep - 1) / kstep;
        long long cols = full_tiles ? tile_n : ((n1 - n0) + 31) / 32 * 32;
        total += 2.0 * (double)g.M * (double)cols * ((double)(steps * kstep) * g.KH + bias_k);
    }
    return total;
}

// MFMA flops a walk of geometry g issues on the kernel that serves it (the same routing as the
// launch: a plan on the streaming kernel runs its dense walk on the LDS-staged variant where that
// fits, else on the largest streaming instance, else on the tiled kernel).
static double walk_flops(int plan_kernel, ConvGeom g, int band, foldconv_dtype_t dtype) {
    g.band = band;
    const bool f32 = dtype == FOLDCONV_F32;
    const int align = fc_band_align(plan_kernel, g);
    if (plan_kernel == FC_KERNEL_GATHER) return issued_flops(g, band, 32, f32 ? 2 : 16, 1, false, 0);
    // the vector kernels walk K in steps of two operand chunks: 16 elements of a 16-bit type (8 where the
    // chunks are 8 bytes), 8 of fp32 (there as four MFMAs of K = 2)
    const int kstep = 2 * g.epc;
    if (plan_kernel == FC_KERNEL_STREAM) {
        StreamShape sh;
        if (!band && fc_stream_lds_ok(g)) return issued_flops(g, 0, 64, kstep, align, false, 0);  // bias added in fp32
        // the rank-1 bias product: one MFMA of the K-step's width, or one of K = 2 for fp32
        if (fc_stream_shape(g, band, &sh)) return issued_flops(g, band, 32 * sh.nt, kstep, align, false, f32 ? 2 : kstep);
        // where the tiled kernel does not serve the layer, a dense walk too long for the streaming instances
        // runs the gather kernel
        if (!fc_tiled_ok(g)) return issued_flops(g, band, 32, f32 ? 2 : 16, 1, false, 0);
    }
    return issued_flops(g, band, fc_tiled_bn(g), kstep, align, true, 16);
}

// Fold-factor cost model (paper: the "lightweight cost model" of the MLIR section, in terms of
// channel size, tile alignment and arithmetic intensity): estimated time of one band-walk
// convolution on the kernel the plan routes to,
//     launch-and-drain overhead + max(memory time, matrix time) + filter term,
// with the rates these kernels sustain on MI355X (fitted to the timings of every legal power-of-two
// fold factor of the benchmark layers, rotating buffers, graph replay):
//   * memory: x + y + filter bytes at 6.2 TB/s (of the 8 TB/s HBM peak), 7.0 TB/s for launches of the streaming
//     kernel long enough to pace their store stream (64 MB and more); 5 % less with 8-byte operand chunks.  On the streaming kernel a wave
//     owns 64 (or 128) output columns, so y counts at F*C_out rounded up to whole waves: idle
//     lanes store nothing but take their turn (tile alignment);
//   * matrix: issued MFMA flops (band walk, tile padding and the rank-1 bias product included) at
//     1.0 PFLOP/s on the streaming kernel and 0.85 PFLOP/s on the tiled kernel (of the 2.5 PFLOP/s
//     16-bit peak; what the clock management leaves to real operands), 0.05 PFLOP/s on the
//     element-gather kernel that serves fp32 and channel counts off the 16-byte chunk alignment;
//   * filter term: the expanded filter read at 1 TB/s (every wave fetches its own fragments; a larger
//     F buys nothing once F*C_in is aligned, and its F^2 larger filter is not free);
//   * overhead: 4.5 us (streaming), 8 us (tiled), 10 us (gather) per launch.
constexpr double kStreamFp32Rate = 0.08e15;  // issued fp32 MFMA flops per second the streaming kernel sustains

static double model_seconds(const foldconv_shapes_t &s, int wave_columns, bool half_chunks) {
    const double x = (double)s.x_bytes, y = (double)s.y_bytes;
    const double wf = s.prefer_compact ? (double)s.filter_compact_bytes : (double)s.w_exp_bytes;
    double hbm = (s.conv_kernel == FC_KERNEL_STREAM && x + y >= 64e6) ? 7.0e12 : 6.2e12;
    if (half_chunks) hbm *= 0.95;  // twice the load instructions and MFMAs per K value: 69 against 66 us on the 411 MB layer
    double overhead, rate, y_eff = y;
    if (s.conv_kernel == FC_KERNEL_STREAM) {
        overhead = 4.5e-6;
        // fp32: K = 2 MFMAs, 157 TFLOP/s peak; 8-byte operand chunks: K = 8 MFMAs at half the rate of K = 16
        // (0.19 PFLOP/s measured on the guarded nine-step instance, 0.35 and more on the exact two-step one)
        rate = s.dtype == FOLDCONV_F32 ? kStreamFp32Rate : half_chunks ? 0.33e15 : 1.0e15;
        const double cols = (double)((s.Co_fold + wave_columns - 1) / wave_columns) * wave_columns;
        y_eff = y * cols / (double)s.Co_fold;
    } else if (s.conv_kernel == FC_KERNEL_TILED) {
        overhead = 8e-6;
        rate = 0.85e15;
    } else {
        overhead = 10e-6;
        rate = s.dtype == FOLDCONV_F32 ? 0.012e15 : 0.05e15;
    }
    const double t_mem = (x + y_eff + wf) / hbm;
    const double t_mma = s.issued_flops_band / rate;
    return overhead + (t_mem > t_mma ? t_mem : t_mma) + wf / 1e12;
}

extern "C" int foldconv_plan(int N, int H, int W, int C_in, int C_out, int KH, int KW, int pad,
                             int fold_factor, foldconv_dtype_t dtype, foldconv_plan_t *out) {
    if (!out) return FOLDCONV_ERR_BADARG;
    *out = nullptr;
    if (N <= 0 || H <= 0 || W <= 0 || C_in <= 0 || C_out <= 0 || KH <= 0 || KW <= 0 || pad < 0 ||
        fold_factor <= 0)
        return FOLDCONV_ERR_BADARG;
    if (dtype != FOLDCONV_F32 && dtype != FOLDCONV_F16 && dtype != FOLDCONV_BF16)
        return FOLDCONV_ERR_BADARG;
    const int F = fold_factor;
    if (W % F != 0) return FOLDCONV_ERR_INDIVISIBLE;  // Algorithm 1 guard

    const int pad_h = KH > 1 ? pad : 0;
    const int pad_w = KW > 1 ? pad : 0;
    const long long H_out = (long long)H + 2 * pad_h - KH + 1;
    const long long W_out = (long long)W + 2 * pad_w - KW + 1;
    if (H_out <= 0 || W_out <= 0) return FOLDCONV_ERR_UNSUPPORTED;

    const int eb = dtype == FOLDCONV_F32 ? 4 : 2;
    const long long Wf = W / F;
    const long long FC = (long long)F * C_in;
    const long long FCo = (long long)F * C_out;
    const long long d_min = floor_div_ll(-(long long)pad_w, F);
    const long long d_max = floor_div_ll((long long)F + KW - 2 - pad_w, F);
    const long long KWf = d_max - d_min + 1;
    const long long Wf_out = (W_out + F - 1) / F;
    const long long M = (long long)N * H_out * Wf_out;
    const long long K = (long long)KH * KWf * FC;
    const int C_pad = (C_in + 7) / 8 * 8;  // the alignment the paper names for fp16 tensor cores
    // The reference path pads the output channels of 16-bit layers the same way, so that it runs the
    // vector kernels too (an unfolded output with C_out off the 16-byte chunk alignment would
    // otherwise fall to the element-gather kernel); the padded result is cropped by a copy.
    const int Co_pad = eb == 2 ? (C_out + 7) / 8 * 8 : C_out;

    // Limits of the kernels' 32-bit tile arithmetic.
    const long long lim = (long long)INT_MAX / 4;
    const long long M_pad = (long long)N * H_out * W_out;
    if (Wf * FC > lim || FCo * Wf_out > lim || K > lim || KWf * FC > lim || M > lim * 2 || M_pad > lim * 2 ||
        (long long)W * C_pad > lim || (long long)KH * KW * C_pad > lim)
        return FOLDCONV_ERR_UNSUPPORTED;

    foldconv_plan_s *p = new (std::nothrow) foldconv_plan_s;
    if (!p) return FOLDCONV_ERR_BADARG;
    memset(p, 0, sizeof(*p));
    p->magic = FOLDCONV_MAGIC;
    foldconv_shapes_t &s = p->s;
    s.N = N; s.H = H; s.W = W; s.C_in = C_in; s.C_out = C_out; s.KH = KH; s.KW = KW; s.pad = pad;
    s.F = F; s.dtype = (int)dtype; s.pad_h = pad_h; s.pad_w = pad_w;
    s.W_fold = (int)Wf; s.C_fold = (int)FC; s.Co_fold = (int)FCo;
    s.d_min = (int)d_min; s.d_max = (int)d_max; s.KW_fold = (int)KWf;
    s.pad_left_fold = (int)-d_min;
    s.pad_right_fold = (int)(Wf_out - Wf + d_min + KWf - 1);
    s.H_out = (int)H_out; s.W_out = (int)W_out; s.W_out_fold = (int)Wf_out;
    s.unfold_is_alias = (W_out == Wf_out * F) ? 1 : 0;
    s.C_pad = C_pad; s.C_out_pad = Co_pad; s.elem_bytes = eb;
    s.gemm_M = M; s.gemm_N = FCo; s.gemm_K = K;
    s.x_bytes = (long long)N * H * W * C_in * eb;
    s.w_bytes = (long long)KH * KW * C_in * C_out * eb;
    s.bias_bytes = (long long)C_out * eb;
    s.w_exp_bytes = K * FCo * eb;
    s.y_bytes = (long long)N * H_out * W_out * C_out * eb;
    s.y_fold_bytes = M * FCo * eb;
    s.useful_flops = 2.0 * (double)N * H_out * W_out * C_out * KH * KW * C_in;

    ConvGeom &g = p->fold;
    g.N = N; g.H = H; g.Hout = (int)H_out; g.Wf = (int)Wf; g.Wf_out = (int)Wf_out;
    g.FC = (int)FC; g.NCo = (int)FCo; g.Co = C_out; g.C = C_in; g.F = F; g.KH = KH; g.KW = KW;
    g.pad_h = pad_h; g.pad_w = pad_w;
    g.e_min = (int)(d_min * FC); g.e_max = (int)((d_max + 1) * FC); g.kwin = g.e_max - g.e_min;
    g.in_row = (int)(Wf * FC); g.out_row = (int)(W_out * C_out); g.M = M;
    g.eb = eb;
    auto set_chunk = [&](ConvGeom &gg, int epc) {
        gg.epc = epc;
        gg.cgcd = fc_gcd_chunk(C_in, epc);
        gg.cJ = (epc - gg.cgcd + KW * C_in + epc - 1) / epc;
    };
    // operand chunks of 16 bytes; 8-byte chunks for a 16-bit layer whose folded channel count allows no more
    set_chunk(g, (eb == 2 && FC % 8 != 0 && FC % 4 == 0) ? 4 : 16 / eb);
    if (eb == 4) {
        // A large fp32 layer is bound by its MFMAs (K = 2 each), and there the chunk that walks fewer structural
        // zeros wins: 8-byte chunks round the band of an output slot to 2 channels and K-steps of 4 instead of
        // 4 and 8 (the headline shape in fp32: 174 us against 191 us).  Layers that the model's rates put on the
        // memory side, the launch-bound ones included, keep 16-byte chunks: fewer load instructions.
        ConvGeom g2 = g;
        set_chunk(g2, 2);
        const bool s4 = fc_choose_kernel(g, dtype) == FC_KERNEL_STREAM;
        const bool s2 = fc_choose_kernel(g2, dtype) == FC_KERNEL_STREAM;
        if (s2 && !s4) {
            g = g2;
        } else if (s2) {
            const double f4 = walk_flops(FC_KERNEL_STREAM, g, 1, dtype), f2 = walk_flops(FC_KERNEL_STREAM, g2, 1, dtype);
            const double t_mem = ((double)s.x_bytes + (double)s.y_bytes) / 6.2e12 + 4.5e-6;
            if (f2 < f4 && f4 / kStreamFp32Rate > t_mem) g = g2;
        }
    }

    // Zero-padded reference problem: F = 1, every pixel C_pad channels.
    ConvGeom &q = p->padc;
    q.N = N; q.H = H; q.Hout = (int)H_out; q.Wf = W; q.Wf_out = (int)W_out;
    q.FC = C_pad; q.NCo = Co_pad; q.Co = Co_pad; q.C = C_pad; q.F = 1; q.KH = KH; q.KW = KW;
    q.pad_h = pad_h; q.pad_w = pad_w;
    q.e_min = -pad_w * C_pad; q.e_max = (KW - pad_w) * C_pad; q.kwin = q.e_max - q.e_min;
    q.in_row = W * C_pad; q.out_row = (int)(W_out * Co_pad); q.M = M_pad;
    q.eb = eb; q.epc = 16 / eb;
    q.cgcd = q.epc; q.cJ = KW * C_pad / q.epc;

    s.conv_kernel = fc_choose_kernel(g, dtype);
    if (W_out != Wf_out * F) {
        // FOLDCONV_FLAG_KEEP_FOLDED stores rows of Wf_out*F*C_out elements instead of W_out*C_out: the
        // kernel (and its 32-bit limits) must hold for both, the more general kernel wins
        ConvGeom gk = g;
        gk.out_row = (int)(Wf_out * FCo);
        const int k2 = fc_choose_kernel(gk, dtype);
        if (k2 < s.conv_kernel) s.conv_kernel = k2;
    }
    s.padded_kernel = fc_choose_kernel(q, dtype);
    {
        ConvGeom gn = g;  // the streaming kernel's channels-first variant sees W_out as the stored row
        gn.out_row = (int)W_out;
        int ks = 0;
        s.out_nchw_fused = (s.conv_kernel == FC_KERNEL_STREAM && fc_stream_nchw_ok(gn, 1, false, &ks)) ? 1 : 0;
    }

    const long long xpad_bytes = (long long)N * H * W * C_pad * eb;
    const long long wpad_bytes = (long long)KH * KW * C_pad * Co_pad * eb;
    const long long ypad_bytes = Co_pad == C_out ? 0 : (long long)N * H_out * W_out * Co_pad * eb;
    s.workspace_bytes = s.conv_kernel == FC_KERNEL_GATHER ? 0 : (long long)align_up((size_t)s.w_exp_bytes, 256);
    // Compact filter: one zero-padded copy of the KW*C_in x C_out tap matrix per kh and per chunk
    // phase for the vector kernels; the gather kernel reads the original filter as it is.
    s.filter_compact_bytes = (long long)align_up(
        s.conv_kernel == FC_KERNEL_GATHER ? (size_t)s.w_bytes
                                          : (size_t)fc_compact_phases(g) * KH * g.cJ * C_out * (g.epc * eb), 256);
    p->ws_xpad = 0;
    p->ws_wpad = align_up((size_t)xpad_bytes, 256);
    p->ws_wpack = p->ws_wpad + align_up((size_t)wpad_bytes, 256);
    p->ws_bpad = p->ws_wpack + (s.padded_kernel == FC_KERNEL_GATHER ? 0 : align_up((size_t)wpad_bytes, 256));
    p->ws_ypad = p->ws_bpad + align_up((size_t)Co_pad * eb, 256);
    s.padded_workspace_bytes = (long long)(p->ws_ypad + align_up((size_t)ypad_bytes, 256));

    // Both filter forms run the same instructions; what differs is the L2 footprint.  On the tiled
    // kernel a packed band of a few megabytes competes with the input rows for the 4 MB L2 of an
    // XCD, and the compact form (one tap matrix for all slots) measured 10-13 % faster there;
    // below that the packed form wins by as much (its staging loads are always contiguous).
    s.prefer_compact = (s.conv_kernel == FC_KERNEL_TILED && s.w_exp_bytes >= (2LL << 20)) ? 1 : 0;
    s.issued_flops_dense = walk_flops(s.conv_kernel, g, 0, dtype);
    s.issued_flops_band = walk_flops(s.conv_kernel, g, 1, dtype);
    s.issued_flops_padded = walk_flops(s.padded_kernel, q, 1, dtype);
    s.model_seconds = model_seconds(s, fc_band_tile_n(s.conv_kernel, g), eb == 2 && g.epc == 4);

    *out = p;
    return FOLDCONV_OK;
}

extern "C" int foldconv_plan_nchw(int N, int C_in, int H, int W, int C_out, int KH, int KW, int pad,
                                  int fold_factor, int fold_axis, foldconv_dtype_t dtype, foldconv_plan_t *out) {
    if (!out) return FOLDCONV_ERR_BADARG;
    *out = nullptr;
    if (fold_axis != FOLDCONV_FOLD_W && fold_axis != FOLDCONV_FOLD_H) return FOLDCONV_ERR_BADARG;
    // Height folding is width folding of the transposed image: rows and columns, KH and KW trade places.
    const int st = fold_axis == FOLDCONV_FOLD_H
                       ? foldconv_plan(N, W, H, C_in, C_out, KW, KH, pad, fold_factor, dtype, out)
                       : foldconv_plan(N, H, W, C_in, C_out, KH, KW, pad, fold_factor, dtype, out);
    if (st != FOLDCONV_OK) return st;
    (*out)->fold_axis = fold_axis;
    (*out)->s.fold_axis = fold_axis;
    if (fold_axis == FOLDCONV_FOLD_H) {
        // slots of a height fold are neighbours along h; the contiguous axis of y runs across the plan's rows
        ConvGeom gn = (*out)->fold;
        gn.out_row = (*out)->s.W_out;
        int ks = 0;
        (*out)->s.out_nchw_fused = ((*out)->s.conv_kernel == FC_KERNEL_STREAM && fc_stream_nchw_ok(gn, 1, true, &ks)) ? 1 : 0;
    }
    return FOLDCONV_OK;
}

extern "C" int foldconv_plan_gemm(long long M, int K, int N, int fold_factor, foldconv_dtype_t dtype,
                                  foldconv_plan_t *out) {
    if (!out) return FOLDCONV_ERR_BADARG;
    *out = nullptr;
    if (M <= 0 || M > INT_MAX) return M <= 0 ? FOLDCONV_ERR_BADARG : FOLDCONV_ERR_UNSUPPORTED;
    if (fold_factor <= 0) return FOLDCONV_ERR_BADARG;
    if (M % fold_factor != 0) return FOLDCONV_ERR_INDIVISIBLE;
    // paper, "GEMM as a 1x1 Convolution": rows of A are spatial positions with K channels.  A 1x1
    // kernel couples no two positions, so the M rows may be laid out as any H x W image; the
    // synthetic width is taken as F times the largest divisor of M/F that keeps the unfolded
    // width under 65000 pixels (and the folded one at most 16384), short enough for the vector
    // kernels' row arithmetic in the folded and in the zero-padded problem alike.
    const long long Mf = M / fold_factor;
    long long cap = 64999 / fold_factor;
    if (cap > 16384) cap = 16384;
    if (cap < 1) cap = 1;
    long long d = Mf < cap ? Mf : cap;
    while (Mf % d != 0) --d;
    return foldconv_plan(1, (int)(Mf / d), (int)(d * fold_factor), K, N, 1, 1, 0, fold_factor, dtype, out);
}

extern "C" int foldconv_choose_fold(int N, int H, int W, int C_in, int C_out, int KH, int KW, int pad,
                                    foldconv_dtype_t dtype, int *fold_factor) {
    if (!fold_factor) return FOLDCONV_ERR_BADARG;
    *fold_factor = 1;
    double best = -1.0;
    int status = FOLDCONV_ERR_BADARG;
    for (int F = 1; F <= 64; F *= 2) {
        if (W % F != 0) break;
        foldconv_plan_t p = nullptr;
        const int st = foldconv_plan(N, H, W, C_in, C_out, KH, KW, pad, F, dtype, &p);
        if (st != FOLDCONV_OK) {
            if (F == 1) return st;
            continue;
        }
        status = FOLDCONV_OK;
        const double t = p->s.model_seconds;
        if (best < 0.0 || t < best * (1.0 - 1e-9)) {
            best = t;
            *fold_factor = F;
        }
        foldconv_plan_destroy(p);
    }
    return status;
}

extern "C" int foldconv_plan_query(foldconv_plan_t plan, foldconv_shapes_t *out) {
    if (!plan || plan->magic != FOLDCONV_MAGIC || !out) return FOLDCONV_ERR_BADARG;
    *out = plan->s;
    return FOLDCONV_OK;
}

extern "C" void foldconv_plan_destroy(foldconv_plan_t plan) {
    if (!plan || plan->magic != FOLDCONV_MAGIC) return;
    plan->magic = 0;
    delete plan;
}

extern "C" const char *foldconv_strerror(int status) {
    switch (status) {
        case FOLDCONV_OK: return "ok";
        case FOLDCONV_ERR_BADARG: return "bad argument";
        case FOLDCONV_ERR_INDIVISIBLE: return "width is not divisible by the fold factor";
        case FOLDCONV_ERR_UNSUPPORTED: return "unsupported problem (empty output or size beyond kernel limits)";
        case FOLDCONV_ERR_WORKSPACE: return "workspace missing, too small or misaligned";
        case FOLDCONV_ERR_HIP: return "HIP launch failed";
        case FOLDCONV_ERR_SCRATCH: return "the problem needs more scratch than the library's static array holds";
        default: return "unknown status";
    }
}
