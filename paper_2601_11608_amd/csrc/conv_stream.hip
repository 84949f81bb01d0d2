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
    long long MT;  // number of 32-pixel M tiles
    int NG;        // column groups of NT*32 columns
    long long J;   // M tiles in flight = stride of a wave's M-tile walk
    int ksteps;    // 16-wide K-steps per kh actually walked (<= KSM)
};

template <typename TR, int NT, int KHM, int KSM, int OCC>
__global__ void __launch_bounds__(256, OCC)
conv_stream_kernel(ConvGeom g, StreamArgs a, const typename TR::T *__restrict__ x, const u32x4 *__restrict__ wp,
                   const typename TR::T *__restrict__ bias, typename TR::T *__restrict__ y) {
    using T = typename TR::T;
    using Vec = typename TR::Vec;
    constexpr int COLS = 32 * NT;                 // output columns per wave
    constexpr int PITCH = COLS * 2 + 16;          // bytes per LDS row (padded)
    constexpr int CHUNKS = COLS / 8;              // 16-byte chunks per row
    constexpr int SLAB = 32 * PITCH + 32 * 8;     // + per-row {offset/8, room} words
    __shared__ __attribute__((aligned(16))) unsigned char lds_all[4 * SLAB];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int r = lane & 31, hf = lane >> 5;
    unsigned char *slab = lds_all + wave * SLAB;
    unsigned *rowinfo = reinterpret_cast<unsigned *>(slab + 32 * PITCH);

    const long long gw = (long long)blockIdx.x * 4 + wave;
    const int ng = (int)(gw % a.NG);
    const long long j0 = gw / a.NG;
    if (j0 >= a.J) return;  // wave-uniform

    const int n_lo = ng * COLS;
    int e_lo, e_hi;
    fc_band_window(g, n_lo, n_lo + COLS, 8, &e_lo, &e_hi);
    const int q_per_kh = g.kwin / 8;

    // ---- filter fragments, resident for the kernel's lifetime -----------------
    Vec wf[KHM][KSM][NT];
#pragma unroll
    for (int kh = 0; kh < KHM; ++kh)
#pragma unroll
        for (int ks = 0; ks < KSM; ++ks)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int e = e_lo + 16 * ks + 8 * hf;
                const int n = n_lo + 32 * nt + r;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (kh < g.KH && ks < a.ksteps && e < e_hi && n < g.NCo)
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

    // ---- per-tile input fragment loads ---------------------------------------
    Vec xf[KHM][KSM];
    unsigned my_off8, my_room;  // this lane's output row: (element offset)/8 and columns left in the row
    auto load_tile = [&](long long mt, Vec (&dst)[KHM][KSM], unsigned &off8, unsigned &room) {
        const long long m = mt * 32 + r;
        const bool vm = m < g.M;
        const long long mm = vm ? m : 0;
        const int wo = (int)(mm % g.Wf_out);
        const long long rowid = mm / g.Wf_out;
        const int ho = (int)(rowid % g.Hout);
        const long long img = rowid / g.Hout;
        const int e0 = e_lo + 8 * hf;            // this lane's extended channel at K-step 0
        const int col0 = wo * g.FC + e0;         // and its column inside the input row
        const T *base = x + (img * g.H + ho - g.pad_h) * (long long)g.in_row + col0;
        const int oc = wo * g.NCo;
        off8 = (unsigned)((rowid * g.out_row + oc) >> 3);
        room = vm && oc < g.out_row ? (unsigned)(g.out_row - oc) : 0u;
#pragma unroll
        for (int kh = 0; kh < KHM; ++kh) {
            const int hi = ho + kh - g.pad_h;
            const bool rv = vm && kh < g.KH && hi >= 0 && hi < g.H;
#pragma unroll
            for (int ks = 0; ks < KSM; ++ks) {
                const int col = col0 + 16 * ks;
                u32x4 v = {0u, 0u, 0u, 0u};
                // in-bounds: row hi exists, and the 8-element chunk [col, col+8) lies inside it
                // (col and in_row are multiples of 8)
                if (rv && ks < a.ksteps && e0 + 16 * ks < e_hi && col >= 0 && col < g.in_row)
                    v = *reinterpret_cast<const u32x4 *>(base + (long long)kh * g.in_row + 16 * ks);
                dst[kh][ks] = __builtin_bit_cast(Vec, v);
            }
        }
    };

    long long mt = j0;
    load_tile(mt, xf, my_off8, my_room);

    for (; mt < a.MT; mt += a.J) {
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
                if (kh < g.KH && ks < a.ksteps) {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) acc[nt] = TR::mfma(wf[kh][ks][nt], xf[kh][ks], acc[nt]);
                }

        const unsigned cur_off8 = my_off8, cur_room = my_room;
        if (mt + a.J < a.MT) load_tile(mt + a.J, xf, my_off8, my_room);  // prefetch the next tile's input

        // ---- epilogue: ReLU, round, transpose through LDS, row-contiguous stores ----
        if (hf == 0) {
            rowinfo[2 * r] = cur_off8;
            rowinfo[2 * r + 1] = cur_room;
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float v0 = acc[nt][4 * q], v1 = acc[nt][4 * q + 1], v2 = acc[nt][4 * q + 2], v3 = acc[nt][4 * q + 3];
                if (g.relu) {
                    v0 = v0 > 0.0f ? v0 : 0.0f;
                    v1 = v1 > 0.0f ? v1 : 0.0f;
                    v2 = v2 > 0.0f ? v2 : 0.0f;
                    v3 = v3 > 0.0f ? v3 : 0.0f;
                }
                u32x2 pk = {pack2<TR>(v0, v1), pack2<TR>(v2, v3)};
                *reinterpret_cast<u32x2 *>(slab + r * PITCH + (32 * nt + 8 * q + 4 * hf) * 2) = pk;
            }
        wave_lds_sync();
#pragma unroll
        for (int idx0 = 0; idx0 < 32 * CHUNKS; idx0 += 64) {
            const int idx = idx0 + lane;
            const int row = idx / CHUNKS, ch = idx - row * CHUNKS;
            if ((32 * CHUNKS) % 64 == 0 || idx < 32 * CHUNKS) {
                const unsigned off8 = rowinfo[2 * row];
                const unsigned room = rowinfo[2 * row + 1];
                const int n = n_lo + 8 * ch;
                const u32x4 v = *reinterpret_cast<const u32x4 *>(slab + row * PITCH + ch * 16);
                if (n < g.NCo && (unsigned)(n + 8) <= room)
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(y) + ((long long)off8 + (n >> 3)));
            }
        }
        wave_lds_sync();
    }
}

template <typename TR, int NT, int KHM, int KSM, int OCC>
int launch_inst(const ConvGeom &g, int ksteps, const void *x, const void *wp, const void *bias, void *y,
                hipStream_t st) {
    using T = typename TR::T;
    StreamArgs a;
    a.MT = (g.M + 31) / 32;
    a.NG = (g.NCo + 32 * NT - 1) / (32 * NT);
    a.ksteps = ksteps;
    // Persistent grid: OCC workgroups per CU on 256 CUs, rounded so that the
    // wave count is a multiple of NG (each M tile is then finished by NG waves
    // running side by side) and no more tiles in flight than there are tiles.
    long long waves = 256LL * OCC * 4;
    long long J = waves / a.NG;
    if (J < 1) J = 1;
    if (J > a.MT) J = a.MT;
    a.J = J;
    const long long blocks = (J * a.NG + 3) / 4;
    conv_stream_kernel<TR, NT, KHM, KSM, OCC><<<(unsigned)blocks, 256, 0, st>>>(
        g, a, (const T *)x, (const u32x4 *)wp, (const T *)bias, (T *)y);
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
