// Filter-stationary streaming MFMA convolution for layers whose K extent is
// small (the misaligned-C_in layers width folding is meant for).
//
// Such layers are bound by the output write, not by the matrix cores: on the
// 224x224 C_in = 3 first layer the output is 411 MB against 19 MB of input.
// So the kernel is organised around the store stream:
//   * each wave owns NT*32 output columns (n = g*C_out + co) for its whole
//     life and keeps the filter fragments it needs for them in registers:
//     only the K-steps inside the block band of w' for those output slots
//     (paper: Eq. "filter_construct"; off-band blocks are structural zeros),
//     or every K-step when the dense walk is requested;
//   * it then streams 32-pixel M tiles: 16-byte input fragments straight from
//     the (cache-resident) folded input, a handful of MFMAs, bias through one
//     extra rank-1 MFMA (bias x ones) that also initialises the accumulators,
//     ReLU, one rounding to the output type;
//   * the accumulator tile is transposed through a wave-private LDS slab so
//     that every store instruction writes whole rows of the reconstructed
//     output: 16 bytes per lane, consecutive lanes on consecutive addresses.
// Waves never synchronise with each other.
// paper: Eq. "new_conv_H" (folded convolution), Eq. "bias_construct",
// Reconstruct step (fused into the store addressing).
#include <hip/hip_runtime.h>
#include <stdlib.h>

#include "launch.h"
#include "mfma_types.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <typename TR>
__device__ __forceinline__ unsigned pack2(float a, float b);
template <>
__device__ __forceinline__ unsigned pack2<F16Traits>(float a, float b) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 v = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(unsigned, v);
}
template <>
__device__ __forceinline__ unsigned pack2<BF16Traits>(float a, float b) {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    b2 v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(unsigned, v);
}

__device__ __forceinline__ void wave_lds_sync() {
    // Orders this wave's LDS writes before its later LDS reads of other lanes'
    // data (LDS executes a wave's instructions in order; this stops the
    // compiler from moving them and waits for outstanding LDS operations).
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

struct StreamArgs {
    unsigned MT;        // number of 32-pixel M tiles
    unsigned J;         // M tiles in flight = stride of a wave's M-tile walk
    int NG;             // column groups of NT*32 columns
    int ksteps;         // 16-wide K-steps per kh actually walked (<= KSM)
    unsigned dW, dH, dI;  // the walk stride of 32*J pixels as (folded column, row, image) steps
    unsigned mgW, mgH;  // ceil(2^32 / Wf_out), ceil(2^32 / Hout): exact division of small numerators
    unsigned x_bytes;   // extent of x for the range-checked buffer loads
    int linear_out;     // stored rows are exactly Wf_out*NCo long: y offset is m*NCo + n
};

// floor(t / d) for t < d + 64 and d < 65000, with mg = ceil(2^32 / d)
__device__ __forceinline__ unsigned small_div(unsigned t, unsigned mg, unsigned d) {
    return d == 1u ? t : __umulhi(t, mg);
}

// EXACT: g.KH == KHM and a.ksteps == KSM, so the K loops carry no run-time guards.
template <typename TR, int NT, int KHM, int KSM, int OCC, bool EXACT, bool RELU>
__global__ void __launch_bounds__(256, OCC)
conv_stream_kernel(ConvGeom g, StreamArgs a, const typename TR::T *__restrict__ x, const u32x4 *__restrict__ wp,
                   const typename TR::T *__restrict__ bias, typename TR::T *__restrict__ y) {
    using T = typename TR::T;
    using Vec = typename TR::Vec;
    constexpr int COLS = 32 * NT;                 // output columns per wave
    constexpr int PITCH = COLS * 2 + 16;          // bytes per LDS row (padded)
    constexpr int CHUNKS = COLS / 8;              // 16-byte chunks per row
    constexpr int PASSES = (32 * CHUNKS + 63) / 64;
    constexpr int SLAB = 32 * PITCH;
    __shared__ __attribute__((aligned(16))) unsigned char lds_all[4 * SLAB];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, hf = lane >> 5;
    unsigned char *slab = lds_all + wave * SLAB;

    const unsigned gw = blockIdx.x * 4 + wave;
    const int ng = (int)(gw % (unsigned)a.NG);
    const unsigned j0 = gw / (unsigned)a.NG;
    if (j0 >= a.J) return;  // wave-uniform

    const int KH = EXACT ? KHM : g.KH;
    const int KS = EXACT ? KSM : a.ksteps;
    const int n_lo = ng * COLS;
    int e_lo, e_hi;
    fc_band_window(g, n_lo, n_lo + COLS, 8, &e_lo, &e_hi);
    const int q_per_kh = g.kwin / 8;
    const int e0 = e_lo + 8 * hf;  // this lane's extended channel at K-step 0

    // ---- filter fragments, resident for the kernel's lifetime -----------------
    Vec wf[KHM][KSM][NT];
#pragma unroll
    for (int kh = 0; kh < KHM; ++kh)
#pragma unroll
        for (int ks = 0; ks < KSM; ++ks)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int e = e0 + 16 * ks;
                const int n = n_lo + 32 * nt + r;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (kh < KH && ks < KS && e < e_hi && n < g.NCo)
                    v = wp[((long long)kh * q_per_kh + ((e - g.e_min) >> 3)) * g.NCo + n];
                wf[kh][ks][nt] = __builtin_bit_cast(Vec, v);
            }
    // bias enters as a rank-1 MFMA: A = bias in K slot 0, B = 1 in K slot 0
    Vec bf[NT], ones;
#pragma unroll
    for (int i = 0; i < 8; ++i) ones[i] = (T)0.0f;
    if (hf == 0) ones[0] = (T)1.0f;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
        for (int i = 0; i < 8; ++i) bf[nt][i] = (T)0.0f;
        const int n = n_lo + 32 * nt + r;
        if (g.has_bias && hf == 0 && n < g.NCo) bf[nt][0] = bias[n % g.Co];
    }

    // Input fragments come through a range-checked buffer resource: a lane whose
    // fragment lies outside the image (zero padding) uses an offset beyond the
    // extent and receives zeros, with no branch and no select afterwards.
    const __amdgpu_buffer_rsrc_t xr =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<T *>(x), 0, (int)a.x_bytes, 0x00020000);
    constexpr unsigned kOutOfRange = 0x80000000u;

    // ---- the wave's current tile: first pixel m0 = (img0, ho0, wo0), advanced incrementally ----
    unsigned m0 = j0 * 32u;
    unsigned wo0 = m0 % (unsigned)g.Wf_out;
    unsigned ho0, img0;
    {
        const unsigned rowid = m0 / (unsigned)g.Wf_out;
        ho0 = rowid % (unsigned)g.Hout;
        img0 = rowid / (unsigned)g.Hout;
    }
    // K-steps whose chunk lies inside this wave's band window (loop invariant per lane)
    unsigned ksmask = 0;
#pragma unroll
    for (int ks = 0; ks < KSM; ++ks)
        if (ks < KS && e0 + 16 * ks < e_hi) ksmask |= 1u << ks;

    // per-lane constants of the row-wise store phase
    int st_row[PASSES], st_n8[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int idx = p * 64 + lane;
        st_row[p] = idx / CHUNKS;
        st_n8[p] = (n_lo >> 3) + (idx - st_row[p] * CHUNKS);
    }

    u32x4 xf[KHM][KSM];
    auto load_tile = [&](u32x4 (&dst)[KHM][KSM]) {
        const unsigned t = wo0 + (unsigned)r;
        const unsigned q = small_div(t, a.mgW, (unsigned)g.Wf_out);
        const unsigned wo = t - q * (unsigned)g.Wf_out;
        const unsigned hr = ho0 + q;
        const unsigned q2 = small_div(hr, a.mgH, (unsigned)g.Hout);
        const unsigned ho = hr - q2 * (unsigned)g.Hout;
        const unsigned img = img0 + q2;
        const bool vm = m0 + (unsigned)r < (unsigned)g.M;
        const int col0 = (int)wo * g.FC + e0;  // column of K-step 0 inside the input row
        const int pix0 = ((int)(img * (unsigned)g.H + ho) - g.pad_h) * g.in_row + col0;  // element offset in x
        unsigned colok = 0;
#pragma unroll
        for (int ks = 0; ks < KSM; ++ks) {
            const int col = col0 + 16 * ks;
            if (((ksmask >> ks) & 1u) && col >= 0 && col < g.in_row) colok |= 1u << ks;
        }
#pragma unroll
        for (int kh = 0; kh < KHM; ++kh) {
            const int hi = (int)ho + kh - g.pad_h;
            const bool rv = vm && kh < KH && hi >= 0 && hi < g.H;
#pragma unroll
            for (int ks = 0; ks < KSM; ++ks) {
                // in range: row hi exists and the 8-element chunk [col, col+8) lies inside it
                // (col and in_row are multiples of 8)
                const bool ok = rv && ((colok >> ks) & 1u);
                const unsigned voff = ok ? 2u * (unsigned)(pix0 + kh * g.in_row + 16 * ks) : kOutOfRange;
                dst[kh][ks] = __builtin_amdgcn_raw_buffer_load_b128(xr, voff, 0, 0);
            }
        }
    };
    auto advance = [&]() {
        m0 += a.J * 32u;
        wo0 += a.dW;
        unsigned c = wo0 >= (unsigned)g.Wf_out ? 1u : 0u;
        wo0 -= c * (unsigned)g.Wf_out;
        ho0 += a.dH + c;
        c = ho0 >= (unsigned)g.Hout ? 1u : 0u;
        ho0 -= c * (unsigned)g.Hout;
        img0 += a.dI + c;
    };

    load_tile(xf);

    for (unsigned mt = j0; mt < a.MT; mt += a.J) {
        floatx16_t acc[NT];
        floatx16_t zero;
#pragma unroll
        for (int i = 0; i < 16; ++i) zero[i] = 0.0f;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = TR::mfma(bf[nt], ones, zero);
#pragma unroll
        for (int kh = 0; kh < KHM; ++kh)
#pragma unroll
            for (int ks = 0; ks < KSM; ++ks)
                if (EXACT || (kh < KH && ks < KS)) {
                    const Vec xv = __builtin_bit_cast(Vec, xf[kh][ks]);
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) acc[nt] = TR::mfma(wf[kh][ks][nt], xv, acc[nt]);
                }

        // where this tile's rows go (wave-uniform part), then move on and prefetch
        const unsigned cur_m0 = m0, cur_wo0 = wo0, cur_rowid0 = img0 * (unsigned)g.Hout + ho0;
        advance();
        if (mt + a.J < a.MT) load_tile(xf);  // the next tile's input stays in flight across the epilogue

        // ---- epilogue: round, ReLU, transpose through LDS, row-contiguous stores ----
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                u32x2 pk = {pack2<TR>(acc[nt][4 * q], acc[nt][4 * q + 1]), pack2<TR>(acc[nt][4 * q + 2], acc[nt][4 * q + 3])};
                if (RELU) {
                    // max(v, 0) on the rounded 16-bit patterns as signed integers: negative
                    // values (sign bit set) become +0, everything else is unchanged
                    typedef short s16x4 __attribute__((ext_vector_type(4)));
                    const s16x4 z = {0, 0, 0, 0};
                    pk = __builtin_bit_cast(u32x2, __builtin_elementwise_max(__builtin_bit_cast(s16x4, pk), z));
                }
                *reinterpret_cast<u32x2 *>(slab + r * PITCH + (32 * nt + 8 * q + 4 * hf) * 2) = pk;
            }
        wave_lds_sync();
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int row = st_row[p];
            if ((32 * CHUNKS) % 64 == 0 || row < 32) {
                const unsigned mrow = cur_m0 + (unsigned)row;
                const u32x4 v = *reinterpret_cast<const u32x4 *>(slab + row * PITCH + (st_n8[p] - (n_lo >> 3)) * 16);
                bool ok = mrow < (unsigned)g.M && st_n8[p] * 8 < g.NCo;
                unsigned long long off8;
                if (a.linear_out) {
                    off8 = (unsigned long long)mrow * (unsigned)(g.NCo >> 3) + (unsigned)st_n8[p];
                } else {
                    const unsigned t = cur_wo0 + (unsigned)row;
                    const unsigned q = small_div(t, a.mgW, (unsigned)g.Wf_out);
                    const unsigned oc = (t - q * (unsigned)g.Wf_out) * (unsigned)g.NCo + (unsigned)st_n8[p] * 8u;
                    ok = ok && oc + 8u <= (unsigned)g.out_row;
                    off8 = ((unsigned long long)(cur_rowid0 + q) * (unsigned)g.out_row + oc) >> 3;
                }
                if (ok) __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(y) + off8);
            }
        }
        wave_lds_sync();
    }
}

static unsigned magic_for(unsigned d) { return d <= 1 ? 0u : (unsigned)(((1ULL << 32) + d - 1) / d); }

template <typename TR, int NT, int KHM, int KSM, int OCC>
int launch_inst(const ConvGeom &g, int ksteps, const void *x, const void *wp, const void *bias, void *y,
                hipStream_t st) {
    using T = typename TR::T;
    StreamArgs a;
    a.MT = (unsigned)((g.M + 31) / 32);
    a.NG = (g.NCo + 32 * NT - 1) / (32 * NT);
    a.ksteps = ksteps;
    // Persistent grid: as many workgroups as stay resident on 256 CUs (asked
    // of the runtime once per instance), rounded so that the wave count is a
    // multiple of NG (each M tile is then finished by NG waves running side
    // by side) and no more tiles in flight than there are tiles.
    static int resident = 0;  // workgroups per CU; benign race: every thread computes the same value
    if (resident == 0) {
        int nb = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(
                &nb, conv_stream_kernel<TR, NT, KHM, KSM, OCC, true, false>, 256, 0) != hipSuccess || nb < 1)
            nb = OCC;
        resident = nb > 4 ? 4 : nb;
    }
    int per_cu = resident;
    if (const char *e = getenv("FOLDCONV_TUNE_WGS_PER_CU")) per_cu = atoi(e) > 0 ? atoi(e) : per_cu;
    long long waves = 256LL * per_cu * 4;
    long long J = waves / a.NG;
    if (J < 1) J = 1;
    if (J > a.MT) J = a.MT;
    a.J = (unsigned)J;
    const long long S = J * 32, plane = (long long)g.Hout * g.Wf_out;
    a.dI = (unsigned)(S / plane);
    a.dH = (unsigned)((S % plane) / g.Wf_out);
    a.dW = (unsigned)((S % plane) % g.Wf_out);
    a.mgW = magic_for((unsigned)g.Wf_out);
    a.mgH = magic_for((unsigned)g.Hout);
    a.x_bytes = (unsigned)((long long)g.N * g.H * g.in_row * (long long)sizeof(T));
    a.linear_out = g.out_row == g.Wf_out * g.NCo ? 1 : 0;
    const unsigned blocks = (unsigned)((J * a.NG + 3) / 4);
    const bool exact = g.KH == KHM && ksteps == KSM;
#define FC_GO(EX, RL)                                                                       \
    conv_stream_kernel<TR, NT, KHM, KSM, OCC, EX, RL><<<blocks, 256, 0, st>>>(              \
        g, a, (const T *)x, (const u32x4 *)wp, (const T *)bias, (T *)y)
    if (exact && g.relu) FC_GO(true, true);
    else if (exact) FC_GO(true, false);
    else if (g.relu) FC_GO(false, true);
    else FC_GO(false, false);
#undef FC_GO
    return (int)hipGetLastError();
}

template <typename TR>
int launch_shape(const ConvGeom &g, const StreamShape &sh, const void *x, const void *wp, const void *bias, void *y,
                 hipStream_t st) {
    int idx = 0;
#define FC_INST(NT_, KHM_, KSM_, OCC_) \
    if (sh.inst == idx++) return launch_inst<TR, NT_, KHM_, KSM_, OCC_>(g, sh.ksteps, x, wp, bias, y, st);
    FC_STREAM_INSTANCES(FC_INST)
#undef FC_INST
    return (int)hipErrorInvalidValue;
}

}  // namespace

int fc_launch_conv_stream(foldconv_dtype_t dt, const ConvGeom &g, const void *x, const void *w_pack, const void *bias,
                          void *y, void *stream) {
    StreamShape sh;
    if (!fc_stream_shape(g, g.band, &sh)) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    if (dt == FOLDCONV_F16) return launch_shape<F16Traits>(g, sh, x, w_pack, bias, y, st);
    if (dt == FOLDCONV_BF16) return launch_shape<BF16Traits>(g, sh, x, w_pack, bias, y, st);
    return (int)hipErrorInvalidValue;
}
