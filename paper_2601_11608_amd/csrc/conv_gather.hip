// Element-gather MFMA convolution: correct for every shape, dtype and
// alignment; used for fp32 and for channel counts that miss the 16-byte
// chunk alignment (the role Algorithm 1 gives to its fallback branch, except
// that the result is still the folded convolution).  One wave owns one
// 32 (output columns n) x 32 (output pixels m) tile and walks
// K = (kh, extended channel e) straight from global memory; the filter is
// read in its canonical [KH][KW'][F*C_in][F*C_out] layout, or, as compact
// storage, straight from the original [KH][KW][C_in][C_out] filter.
// paper: Eq. "new_conv_H" (folded convolution), Eq. "bias_construct".
#include <hip/hip_runtime.h>

#include "launch.h"
#include "mfma_types.h"

namespace {

template <typename TR>
__global__ void __launch_bounds__(256)
conv_gather_kernel(ConvGeom g, const typename TR::T *__restrict__ x, const typename TR::T *__restrict__ we,
                   const typename TR::T *__restrict__ bias, typename TR::T *__restrict__ y, long long tiles_m,
                   int tiles_n) {
    using T = typename TR::T;
    constexpr int PL = TR::kPerLane;
    constexpr int KS = TR::kStep;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const long long tile = (long long)blockIdx.x * 4 + wave;
    if (tile >= tiles_m * tiles_n) return;  // wave-uniform; the kernel has no barrier
    const long long mt = tile / tiles_n;
    const int nt = (int)(tile - mt * tiles_n);
    const int r = lane & 31, hf = lane >> 5;

    const long long m = mt * 32 + r;
    const bool valid_m = m < g.M;
    const long long mm = valid_m ? m : 0;
    const int wo = (int)(mm % g.Wf_out);
    const long long rowid = mm / g.Wf_out;  // image*Hout + ho
    const int ho = (int)(rowid % g.Hout);
    const long long img = rowid / g.Hout;

    const int n0 = nt * 32;
    const int my_n = n0 + r;
    const bool valid_n = my_n < g.NCo;

    int e_lo, e_hi;
    fc_band_window(g, n0, n0 + 32, 1, &e_lo, &e_hi);

    // Filter entry w'[kh][e - e_min][my_n].  With compact storage `we` is the original filter
    // [KH][KW*C_in][C_out] and the entry is tap row t = e - (g-p)*C_in of output slot g, zero
    // outside [0, KW*C_in) (paper: Eq. "filter_construct", gather form).
    const int slot = (valid_n ? my_n : 0) / g.Co, co = (valid_n ? my_n : 0) - slot * g.Co;
    const int t_off = (slot - g.pad_w) * g.C, taps_c = g.KW * g.C;
    auto filt = [&](int kh, int e) -> T {
        if (g.compact) {
            const int tr = e - t_off;
            return (tr >= 0 && tr < taps_c) ? we[((long long)kh * taps_c + tr) * g.Co + co] : (T)0.0f;
        }
        return we[((long long)kh * g.kwin + (e - g.e_min)) * g.NCo + my_n];
    };

    floatx16_t acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;

    for (int kh = 0; kh < g.KH; ++kh) {
        const int hi = ho + kh - g.pad_h;
        const bool row_ok = valid_m && hi >= 0 && hi < g.H;
        const T *xrow = x + (img * g.H + (row_ok ? hi : 0)) * (long long)g.in_row;
        const int col0 = wo * g.FC;
        for (int e0 = e_lo; e0 < e_hi; e0 += KS) {
            typename TR::Vec a, b;
            if constexpr (PL == 1) {
                const int e = e0 + hf;
                const bool ek = e < e_hi;
                const int col = col0 + e;
                a = (valid_n && ek) ? filt(kh, e) : 0.0f;
                b = (row_ok && ek && col >= 0 && col < g.in_row) ? xrow[col] : 0.0f;
            } else {
#pragma unroll
                for (int j = 0; j < PL; ++j) {
                    const int e = e0 + hf * PL + j;
                    const bool ek = e < e_hi;
                    const int col = col0 + e;
                    a[j] = (valid_n && ek) ? filt(kh, e) : (T)0.0f;
                    b[j] = (row_ok && ek && col >= 0 && col < g.in_row) ? xrow[col] : (T)0.0f;
                }
            }
            acc = TR::mfma(a, b, acc);
        }
    }

    if (!valid_m) return;
    T *yrow = y + rowid * (long long)g.out_row;
    const int ocol0 = wo * g.NCo;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int n = n0 + 8 * (i >> 2) + 4 * hf + (i & 3);
        const int oc = ocol0 + n;
        if (n < g.NCo && oc < g.out_row) {
            float v = acc[i];
            if (g.has_bias) v += (float)bias[n % g.Co];
            if (g.relu) v = v > 0.0f ? v : 0.0f;
            yrow[oc] = TR::from_float(v);
        }
    }
}

template <typename TR>
int launch(const ConvGeom &g, const void *x, const void *we, const void *bias, void *y, hipStream_t st) {
    using T = typename TR::T;
    const long long tiles_m = (g.M + 31) / 32;
    const int tiles_n = (g.NCo + 31) / 32;
    const long long blocks = (tiles_m * tiles_n + 3) / 4;
    if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    conv_gather_kernel<TR><<<(unsigned)blocks, 256, 0, st>>>(g, (const T *)x, (const T *)we, (const T *)bias, (T *)y,
                                                             tiles_m, tiles_n);
    return (int)hipGetLastError();
}

}  // namespace

int fc_launch_conv_gather(foldconv_dtype_t dt, const ConvGeom &g, const void *x, const void *we, const void *bias,
                          void *y, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    switch (dt) {
        case FOLDCONV_F16: return launch<F16Traits>(g, x, we, bias, y, st);
        case FOLDCONV_BF16: return launch<BF16Traits>(g, x, we, bias, y, st);
        default: return launch<F32Traits>(g, x, we, bias, y, st);
    }
}
