/*
 * foldconv_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, fp64 CPU statement of what the width-folding convolution path
 * computes.  Nothing in the product (the HIP library, its Python binding)
 * may call this file; only the tests, the smoke check and the CPU-baseline
 * leg of the benchmark do.  It shares no code with the GPU path.
 *
 * Layouts (row-major, last index fastest):
 *   x  [N][H][W][C]          input, NHWC            (paper: Algorithm 1, REQUIRE)
 *   w  [KH][KW][C][Co]       filter, HWIO           (paper: Algorithm 1, REQUIRE)
 *   b  [Co]                  bias
 *   xf [N][H][W/F][F*C]      folded input           (paper: Eq. "width_fold_def",
 *                                                    and the general-C_in form in
 *                                                    "Width Folding: Mathematical
 *                                                    Perspective")
 *   we [KH][KWf][F*C][F*Co]  expanded filter        (paper: Eq. "filter_construct",
 *                                                    Algorithm 1 "Define W_f'")
 *   bf [F*Co]                replicated bias        (paper: Eq. "bias_construct")
 *
 * Parity pins (tests/test_oracle_*.py): library fp64 cross-correlation,
 * an independent einsum formulation, numpy.kron for the K_W = 1 case
 * (paper: Kronecker remark), hand-worked examples, delta/shift filters,
 * block counts, and planted-mistake sensitivity checks.
 *
 * Readings where the paper is silent (spatial padding, K_W > 1 along the
 * folded axis, ragged output width) are listed in the design document; the
 * paper proves only the K x 1, C_in = 1 case (section "Correctness of Width
 * Folding Transformation"), which is the special case p = 0, K_W = 1 here.
 */
#include <stddef.h>
#include <string.h>

static long floor_div(long a, long b) /* b > 0 */
{
    long q = a / b;
    if ((a % b != 0) && (a < 0)) --q;
    return q;
}

/*
 * Direct cross-correlation (no kernel flip), stride 1, zero padding realised
 * by omitting out-of-range taps:
 *   y[n,ho,wo,co] = b[co] + sum_{kh,kw,c} x[n, ho+kh-pad_top, wo+kw-pad_left, c] * w[kh,kw,c,co]
 * paper: the standard contraction in "Width Folding: Mathematical
 * Perspective"; Eq. "orig_conv_H" is the case KW = 1, C = 1, pads 0.
 * Output extent (H_out, W_out) is given by the caller so the same routine
 * serves symmetric padding (original problem) and the asymmetric width
 * padding of the folded problem.  Each output is summed by one thread in
 * fixed (kh, kw, c) order.
 */
void oracle_conv2d_nhwc(const double *x, const double *w, const double *b, double *y,
                        int N, int H, int W, int C, int Co, int KH, int KW,
                        int pad_top, int pad_left, int H_out, int W_out, int relu)
{
    long rows = (long)N * H_out;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        int n = (int)(r / H_out);
        int ho = (int)(r % H_out);
        for (int wo = 0; wo < W_out; ++wo) {
            double *yo = y + (((size_t)n * H_out + ho) * W_out + wo) * Co;
            for (int co = 0; co < Co; ++co) {
                double acc = b ? b[co] : 0.0;
                for (int kh = 0; kh < KH; ++kh) {
                    int hi = ho + kh - pad_top;
                    if (hi < 0 || hi >= H) continue;
                    for (int kw = 0; kw < KW; ++kw) {
                        int wi = wo + kw - pad_left;
                        if (wi < 0 || wi >= W) continue;
                        const double *xi = x + (((size_t)n * H + hi) * W + wi) * C;
                        const double *wk = w + ((size_t)(kh * KW + kw) * C) * Co + co;
                        for (int c = 0; c < C; ++c)
                            acc += xi[c] * wk[(size_t)c * Co];
                    }
                }
                if (relu && acc < 0.0) acc = 0.0;
                yo[co] = acc;
            }
        }
    }
}

/*
 * Input width fold: xf[n,h,w',f*C+c] = x[n,h,F*w'+f,c].
 * paper: Eq. "width_fold_def" (C = 1) and the c' = f*C_in + c form.
 * Written as the four index loops of Algorithm 1 plus a channel loop.
 */
void oracle_fold_input(const double *x, double *xf, int N, int H, int W, int C, int F)
{
    int Wf = W / F;
    for (int n = 0; n < N; ++n)
        for (int h = 0; h < H; ++h)
            for (int wp = 0; wp < Wf; ++wp)
                for (int f = 0; f < F; ++f)
                    for (int c = 0; c < C; ++c)
                        xf[((((size_t)n * H + h) * Wf + wp) * F + f) * C + c] =
                            x[(((size_t)n * H + h) * W + (F * wp + f)) * C + c];
}

/*
 * Closed forms of the folded problem for symmetric width padding p on the
 * original problem (stride 1).  Output slot g of folded column w' stands for
 * original column F*w'+g; its tap kw reads original column F*w' + (g+kw-p).
 * Writing g+kw-p = F*d + f (0 <= f < F) the tap lands in folded column w'+d,
 * channel block f.  d ranges over [d_min, d_max]:
 *   d_min = floor((0 + 0 - p)/F),  d_max = floor((F-1 + KW-1 - p)/F).
 * For KW = 1, p = 0 (the case the paper proves) d_min = d_max = 0.
 * out[0]=Wf out[1]=d_min out[2]=d_max out[3]=KWf out[4]=W_out out[5]=Wf_out
 * out[6]=pad_left_f out[7]=pad_right_f
 */
void oracle_folded_shapes(int W, int KW, int p, int F, int *out)
{
    int Wf = W / F;
    int d_min = (int)floor_div(-(long)p, F);
    int d_max = (int)floor_div((long)F - 1 + KW - 1 - p, F);
    int KWf = d_max - d_min + 1;
    int W_out = W + 2 * p - KW + 1;
    int Wf_out = (W_out + F - 1) / F;
    out[0] = Wf;
    out[1] = d_min;
    out[2] = d_max;
    out[3] = KWf;
    out[4] = W_out;
    out[5] = Wf_out;
    out[6] = -d_min;                              /* left zero columns of xf   */
    out[7] = Wf_out - Wf + d_min + KWf - 1;       /* right zero columns of xf  */
}

/*
 * Structured filter expansion, in the order the paper gives it: allocate
 * zeros, then copy each original C x Co block to where it belongs.
 * paper: Eq. "filter_construct"; Algorithm 1 ("initialize to zero", then the
 * loop over f copying W_f into diagonal blocks).  For KW = 1, p = 0 this is
 * exactly the block diagonal I_F (x) w.  For taps along the folded axis the
 * block for (output slot g, tap kw) goes to folded tap d - d_min, input
 * block f, with g + kw - p = F*d + f.
 */
void oracle_expand_filter(const double *w, double *we, int KH, int KW, int C, int Co,
                          int F, int p)
{
    int sh[8];
    oracle_folded_shapes(F /* W irrelevant here */, KW, p, F, sh);
    int d_min = sh[1], KWf = sh[3];
    size_t FC = (size_t)F * C, FCo = (size_t)F * Co;
    memset(we, 0, sizeof(double) * (size_t)KH * KWf * FC * FCo);
    for (int g = 0; g < F; ++g)
        for (int kw = 0; kw < KW; ++kw) {
            long t = (long)g + kw - p;
            long d = floor_div(t, F);
            long f = t - d * F;
            for (int kh = 0; kh < KH; ++kh)
                for (int c = 0; c < C; ++c)
                    for (int co = 0; co < Co; ++co)
                        we[(((size_t)kh * KWf + (size_t)(d - d_min)) * FC + (size_t)f * C + c) * FCo +
                           (size_t)g * Co + co] =
                            w[(((size_t)kh * KW + kw) * C + c) * Co + co];
        }
}

/* bf[g*Co+co] = b[co].  paper: Eq. "bias_construct"; Algorithm 1 "Define b'". */
void oracle_tile_bias(const double *b, double *bf, int Co, int F)
{
    for (int g = 0; g < F; ++g)
        for (int co = 0; co < Co; ++co) bf[(size_t)g * Co + co] = b[co];
}

/*
 * Reconstruct: y[n,h,F*w'+g,co] = yf[n,h,w',g*Co+co] for F*w'+g < W_out.
 * paper: "Let w = F w' + f" in the correctness section; the Reconstruct step
 * of the IR formulation.  Columns at or beyond W_out (ragged tail when
 * W_out is not a multiple of F) are dropped.
 */
void oracle_unfold_output(const double *yf, double *y, int N, int H_out, int Wf_out,
                          int F, int Co, int W_out)
{
    for (int n = 0; n < N; ++n)
        for (int h = 0; h < H_out; ++h)
            for (int wp = 0; wp < Wf_out; ++wp)
                for (int g = 0; g < F; ++g) {
                    int wo = F * wp + g;
                    if (wo >= W_out) continue;
                    for (int co = 0; co < Co; ++co)
                        y[(((size_t)n * H_out + h) * W_out + wo) * Co + co] =
                            yf[((((size_t)n * H_out + h) * Wf_out + wp) * F + g) * Co + co];
                }
}

/* Zero-pad the channel axis: xp[..., c] = x[..., c] for c < C, else 0.
 * paper: the zero-padding alternative described in "Difference from Channel
 * Zero-Padding". */
void oracle_pad_channels(const double *x, double *xp, size_t pixels, int C, int C_pad)
{
    for (size_t i = 0; i < pixels; ++i)
        for (int c = 0; c < C_pad; ++c) xp[i * C_pad + c] = (c < C) ? x[i * C + c] : 0.0;
}

/* ------------------------------------------------------------------------
 * Height folding for channels-first tensors (paper: Introduction, "width
 * folding for input in NHWC format (alternatively height folding for NCHW
 * format)").  The same rewrite with the roles of H and W exchanged:
 *   x   [N][C][H][W]            input, NCHW
 *   w   [Co][C][KH][KW]         filter, OIHW
 *   xh  [N][F*C][H/F][W]        height-folded input,  xh[n,f*C+c,h',w] = x[n,c,F*h'+f,w]
 *   wh  [F*Co][F*C][KHf][KW]    expanded filter,
 *         wh[g*Co+co, f*C+c, d-d_min, kw] = w[co,c,F*d+f-g+p,kw]  (tap index in [0,KH), else 0)
 *   yh  [N][F*Co][H'_out][W_out]   folded output, yh[n,g*Co+co,h',w] = y[n,co,F*h'+g,w]
 * The closed forms (d_min, d_max, KHf, pads) are oracle_folded_shapes() with
 * H, KH in the places of W, KW.
 * ------------------------------------------------------------------------ */

/* Direct cross-correlation on channels-first tensors, stride 1, zero padding
 * by omitting out-of-range taps; output extent given by the caller (as in
 * oracle_conv2d_nhwc) so it also serves the asymmetric height padding of the
 * folded problem.  Fixed (c, kh, kw) summation order per output. */
void oracle_conv2d_nchw(const double *x, const double *w, const double *b, double *y,
                        int N, int C, int H, int W, int Co, int KH, int KW,
                        int pad_top, int pad_left, int H_out, int W_out, int relu)
{
    long planes = (long)N * Co;
#pragma omp parallel for schedule(static)
    for (long q = 0; q < planes; ++q) {
        int n = (int)(q / Co), co = (int)(q % Co);
        for (int ho = 0; ho < H_out; ++ho)
            for (int wo = 0; wo < W_out; ++wo) {
                double acc = b ? b[co] : 0.0;
                for (int c = 0; c < C; ++c)
                    for (int kh = 0; kh < KH; ++kh) {
                        int hi = ho + kh - pad_top;
                        if (hi < 0 || hi >= H) continue;
                        for (int kw = 0; kw < KW; ++kw) {
                            int wi = wo + kw - pad_left;
                            if (wi < 0 || wi >= W) continue;
                            acc += x[(((size_t)n * C + c) * H + hi) * W + wi] *
                                   w[(((size_t)co * C + c) * KH + kh) * KW + kw];
                        }
                    }
                if (relu && acc < 0.0) acc = 0.0;
                y[(((size_t)n * Co + co) * H_out + ho) * W_out + wo] = acc;
            }
    }
}

/* xh[n,f*C+c,h',w] = x[n,c,F*h'+f,w]: whole rows of W elements move. */
void oracle_fold_input_h_nchw(const double *x, double *xh, int N, int C, int H, int W, int F)
{
    int Hf = H / F;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int hp = 0; hp < Hf; ++hp)
                for (int f = 0; f < F; ++f)
                    for (int wi = 0; wi < W; ++wi)
                        xh[(((size_t)n * F * C + (size_t)f * C + c) * Hf + hp) * W + wi] =
                            x[(((size_t)n * C + c) * H + (F * hp + f)) * W + wi];
}

/* Zeros, then each original (co, c) tap column copied to its place: output
 * slot g, tap kh lands in folded tap d, input block f with g + kh - p = F*d + f. */
void oracle_expand_filter_h_oihw(const double *w, double *wh, int Co, int C, int KH, int KW,
                                 int F, int p)
{
    int sh[8];
    oracle_folded_shapes(F, KH, p, F, sh);
    int d_min = sh[1], KHf = sh[3];
    size_t FC = (size_t)F * C;
    memset(wh, 0, sizeof(double) * (size_t)F * Co * FC * KHf * KW);
    for (int g = 0; g < F; ++g)
        for (int kh = 0; kh < KH; ++kh) {
            long t = (long)g + kh - p;
            long d = floor_div(t, F);
            long f = t - d * F;
            for (int co = 0; co < Co; ++co)
                for (int c = 0; c < C; ++c)
                    for (int kw = 0; kw < KW; ++kw)
                        wh[((((size_t)g * Co + co) * FC + (size_t)f * C + c) * KHf + (size_t)(d - d_min)) * KW + kw] =
                            w[(((size_t)co * C + c) * KH + kh) * KW + kw];
        }
}

/* y[n,co,F*h'+g,w] = yh[n,g*Co+co,h',w] for F*h'+g < H_out. */
void oracle_unfold_output_h_nchw(const double *yh, double *y, int N, int Co, int Hf_out, int W_out,
                                 int F, int H_out)
{
    for (int n = 0; n < N; ++n)
        for (int g = 0; g < F; ++g)
            for (int co = 0; co < Co; ++co)
                for (int hp = 0; hp < Hf_out; ++hp) {
                    int ho = F * hp + g;
                    if (ho >= H_out) continue;
                    for (int wi = 0; wi < W_out; ++wi)
                        y[(((size_t)n * Co + co) * H_out + ho) * W_out + wi] =
                            yh[(((size_t)n * F * Co + (size_t)g * Co + co) * Hf_out + hp) * W_out + wi];
                }
}
