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
// The element type and the operand chunk are template parameters (the MFMA traits).
// Both operands are read in chunks of E K-contiguous elements, and a K-step is two
// chunks, one per half of the wave: 16-byte chunks and one 32x32x16 MFMA for the
// 16-bit types; 8-byte chunks and one 32x32x8 MFMA for 16-bit layers whose F*C_in
// is a multiple of 4 only; 16-byte chunks and four chained 32x32x2 MFMAs for fp32
// (whose K index inside the step is a permutation of the chunk order, the same one
// for both operands, so the sum is unchanged), or 8-byte chunks and two such MFMAs
// where that walks fewer structural zeros.  Stores are 16 bytes in every case.
// paper: Eq. "new_conv_H" (folded convolution), Eq. "bias_construct",
// Reconstruct step (fused into the store addressing).
#include <hip/hip_runtime.h>
#include <type_traits>

#include "launch.h"
#include "mfma_types.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <typename T>  // two results rounded to the 16-bit output type
__device__ __forceinline__ unsigned pack2(float a, float b);
template <>
__device__ __forceinline__ unsigned pack2<_Float16>(float a, float b) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 v = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(unsigned, v);
}
template <>
__device__ __forceinline__ unsigned pack2<__bf16>(float a, float b) {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    b2 v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(unsigned, v);
}

__device__ __forceinline__ void wave_lds_sync() {
    // A wave's LDS instructions execute in issue order, so data one lane wrote is visible to
    // the other lanes' later reads without any wait.  All that is needed is to keep the
    // compiler from moving LDS accesses across this point.
    __builtin_amdgcn_wave_barrier();
    asm volatile("" ::: "memory");
}

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

struct StreamArgs {
    unsigned MT;        // number of 32-pixel M tiles
    FcDeal deal;        // how M tiles are dealt to the XCDs; deal.stride is the stride of a wave's M-tile walk
    int NG;             // column groups of NT*32 columns
    int ksteps;         // 16-wide K-steps per kh actually walked (<= KSM)
    unsigned dW, dH, dI;  // the walk stride of 32*stride pixels as (folded column, row, image) steps
    unsigned mgW, mgH;  // ceil(2^32 / Wf_out), ceil(2^32 / Hout): exact division of small numerators
    unsigned x_bytes;   // extent of x for the range-checked buffer loads
    int linear_out;     // stored rows are exactly Wf_out*NCo long: y offset is m*NCo + n
    unsigned pace;      // wall-clock ticks * 256 between a wave's store bursts, 0 = unpaced (see launch_inst)
};

// floor(t / d) for t < d + 64 and d < 65000, with mg = ceil(2^32 / d)
__device__ __forceinline__ unsigned small_div(unsigned t, unsigned mg, unsigned d) {
    return d == 1u ? t : __umulhi(t, mg);
}

// EXACT: g.KH == KHM and a.ksteps == KSM, so the K loops carry no run-time guards.
template <typename TR, int NT, int KHM, int KSM, int OCC, bool EXACT, bool RELU>
__global__ void __launch_bounds__(256, OCC)
conv_stream_kernel(ConvGeom g, StreamArgs a, const typename TR::T *__restrict__ x, const typename TR::Vec *__restrict__ wp,
                   const typename TR::T *__restrict__ bias, typename TR::T *__restrict__ y) {
    using T = typename TR::T;
    using Vec = typename TR::Vec;
    constexpr int EB = (int)sizeof(T);            // bytes per element
    constexpr int E = TR::kPerLane;               // elements per operand chunk (g.epc): a K-step is two chunks,
                                                  // one per half of the wave
    constexpr int ESH = E == 8 ? 3 : E == 4 ? 2 : 1;  // log2(E)
    constexpr int CB = E * EB;                    // bytes per operand chunk: 16, or 8 (16-bit types with E = 4, fp32 with E = 2)
    using XV = std::conditional_t<CB == 16, u32x4, u32x2>;  // an input fragment as loaded
    static_assert(sizeof(Vec) == CB && (CB == 16 || CB == 8), "operand chunks of 8 or 16 bytes");
    constexpr int EO = 16 / EB;                   // elements per 16-byte chunk of the stored output
    constexpr int COLS = 32 * NT;                 // output columns per wave
    constexpr int PITCH = COLS * EB + 16;         // bytes per LDS row (padded)
    constexpr int CHUNKS = COLS / EO;             // 16-byte chunks per row
    constexpr int PASSES = (32 * CHUNKS + 63) / 64;
    constexpr int SLAB = 32 * PITCH;
    __shared__ __attribute__((aligned(16))) unsigned char lds_all[4 * SLAB];

    constexpr unsigned kOutOfRange = 0x80000000u;  // beyond any resource extent used here
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, hf = lane >> 5;
    unsigned char *slab = lds_all + wave * SLAB;

    // Workgroups are dealt round-robin to the 8 XCDs; M tiles follow them in chunks (FcDeal).
    const unsigned part = blockIdx.x % a.deal.parts;
    const unsigned gw = (blockIdx.x / a.deal.parts) * 4 + wave;
    const int ng = (int)(gw % (unsigned)a.NG);
    const unsigned j0 = gw / (unsigned)a.NG;
    if (j0 >= a.deal.J) return;  // wave-uniform
    const unsigned t_first = fc_deal_first_tile(a.deal, part, j0);  // the wave's first tile

    const int KH = EXACT ? KHM : g.KH;
    const int KS = EXACT ? KSM : a.ksteps;
    const int n_lo = ng * COLS;
    int e_lo, e_hi;
    fc_band_window(g, n_lo, n_lo + COLS, E, &e_lo, &e_hi);
    const int q_per_kh = g.kwin >> ESH;
    const int e0 = e_lo + E * hf;  // this lane's extended channel at K-step 0

    // ---- filter fragments, resident for the kernel's lifetime -----------------
    Vec wf[KHM][KSM][NT];
#pragma unroll
    for (int kh = 0; kh < KHM; ++kh)
#pragma unroll
        for (int ks = 0; ks < KSM; ++ks)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int e = e0 + 2 * E * ks;
                const int n = n_lo + 32 * nt + r;
                Vec v;
#pragma unroll
                for (int i = 0; i < E; ++i) v[i] = (T)0.0f;
                if (kh < KH && ks < KS && e < e_hi && n < g.NCo) {
                    const int q = (e - g.e_min) >> ESH;  // e >= e_min, both multiples of E
                    const long long ci = g.compact ? fc_compact_chunk<E>(g, kh, q, n)
                                                   : ((long long)kh * q_per_kh + q) * g.NCo + n;
                    if (ci >= 0) v = wp[ci];  // off-band chunks of the compact form are zeros
                }
                wf[kh][ks][nt] = v;
            }
    // bias enters as a rank-1 MFMA: A = bias in K slot 0, B = 1 in K slot 0
    Vec bf[NT], ones;
#pragma unroll
    for (int i = 0; i < E; ++i) ones[i] = (T)0.0f;
    if (hf == 0) ones[0] = (T)1.0f;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
        for (int i = 0; i < E; ++i) bf[nt][i] = (T)0.0f;
        const int n = n_lo + 32 * nt + r;
        if (g.has_bias && hf == 0 && n < g.NCo) bf[nt][0] = bias[n % g.Co];
    }

    // Input fragments come through a range-checked buffer resource: a lane whose
    // fragment lies outside the image (zero padding) uses an offset beyond the
    // extent and receives zeros, with no branch and no select afterwards.
    // The loads are issued from inline assembly and waited for with explicit counts (see the
    // loop head): the compiler's own wait insertion would make every wave wait for its
    // previous tile's stores before touching the next tile's input.
    u32x4 xr;
    {
        const unsigned long long xa = (unsigned long long)x;
        xr[0] = (unsigned)xa;
        xr[1] = (unsigned)(xa >> 32) & 0xffffu;  // stride 0: raw buffer, byte offsets
        xr[2] = a.x_bytes;
        xr[3] = 0x00020000u;
        xr[0] = __builtin_amdgcn_readfirstlane(xr[0]);
        xr[1] = __builtin_amdgcn_readfirstlane(xr[1]);
        xr[2] = __builtin_amdgcn_readfirstlane(xr[2]);
        xr[3] = __builtin_amdgcn_readfirstlane(xr[3]);
    }

    // ---- the wave's current tile: first pixel m0 = (img0, ho0, wo0), advanced incrementally ----
    unsigned m0 = t_first * 32u;
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
        if (ks < KS && e0 + 2 * E * ks < e_hi) ksmask |= 1u << ks;

    // per-lane constants of the row-wise store phase: LDS byte offset of the lane's 16-byte
    // chunk in each pass and, when stored rows are contiguous (linear_out), its byte offset
    // from the tile's first output element
    int st_row[PASSES], st_col[PASSES], st_lds[PASSES];
    unsigned st_lin[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int idx = p * 64 + lane;
        st_row[p] = idx / CHUNKS;
        const int ch = idx - st_row[p] * CHUNKS;
        st_col[p] = n_lo + EO * ch;  // first output column of the chunk
        const bool in = st_row[p] < 32 && st_col[p] < g.NCo;
        st_lds[p] = (in ? st_row[p] : 0) * PITCH + ch * 16;
        st_lin[p] = in ? (unsigned)EB * ((unsigned)st_row[p] * (unsigned)g.NCo + (unsigned)st_col[p]) : kOutOfRange;
    }
    const unsigned long long y_rows_total = (unsigned long long)g.N * (unsigned)g.Hout;

    // Store pacing: the wave's next store burst is not issued before this time (ticks * 256).
    unsigned long long pace_next = a.pace ? (unsigned long long)wall_clock64() << 8 : 0ull;

    XV xf[KHM][KSM];
    auto load_tile = [&](XV (&dst)[KHM][KSM]) {
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
            const int col = col0 + 2 * E * ks;
            if (((ksmask >> ks) & 1u) && col >= 0 && col < g.in_row) colok |= 1u << ks;
        }
#pragma unroll
        for (int kh = 0; kh < KHM; ++kh) {
            const int hi = (int)ho + kh - g.pad_h;
            const bool rv = vm && kh < KH && hi >= 0 && hi < g.H;
#pragma unroll
            for (int ks = 0; ks < KSM; ++ks) {
                // in range: row hi exists and the chunk [col, col+E) lies inside it
                // (col and in_row are multiples of E)
                const bool ok = rv && ((colok >> ks) & 1u);
                const unsigned voff = ok ? (unsigned)EB * (unsigned)(pix0 + kh * g.in_row + 2 * E * ks) : kOutOfRange;
                if constexpr (CB == 16)
                    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(dst[kh][ks]) : "v"(voff), "s"(xr) : "memory");
                else
                    asm volatile("buffer_load_dwordx2 %0, %1, %2, 0 offen" : "=v"(dst[kh][ks]) : "v"(voff), "s"(xr) : "memory");
            }
        }
    };
    auto advance = [&]() {
        m0 += a.deal.stride * 32u;
        wo0 += a.dW;
        unsigned c = wo0 >= (unsigned)g.Wf_out ? 1u : 0u;
        wo0 -= c * (unsigned)g.Wf_out;
        ho0 += a.dH + c;
        c = ho0 >= (unsigned)g.Hout ? 1u : 0u;
        ho0 -= c * (unsigned)g.Hout;
        img0 += a.dI + c;
    };

    // Nothing the compiler tracks may be in flight when the hand-counted loads start.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    load_tile(xf);
    // Drain the first tile's loads here: the loop head then only ever waits for loads that were
    // issued ahead of PASSES stores of the previous tile, and leaves those stores in flight.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    for (unsigned mt = t_first; mt < a.MT; mt += a.deal.stride) {
        floatx16_t acc[NT];
        floatx16_t zero;
#pragma unroll
        for (int i = 0; i < 16; ++i) zero[i] = 0.0f;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = TR::mfma_k0(bf[nt], ones, zero);
        if (!EXACT) {
            // Instances with run-time K guards drain every fragment load here, ahead of the guards:
            // a fragment whose K-step is guarded off is never waited for below, and its registers
            // must not be handed to anything else while its load is still in flight.
#pragma unroll
            for (int i = 0; i < KHM * KSM; ++i)
                asm volatile("s_waitcnt vmcnt(0)" : "+v"(xf[i / KSM][i % KSM]) : : "memory");
        }
        static_for<0, KHM * KSM>([&](auto step) {
            constexpr int idx = decltype(step)::value;
            constexpr int kh = idx / KSM, ks = idx % KSM;
            if (EXACT || (kh < KH && ks < KS)) {
                // Vector-memory operations retire in issue order.  Behind this fragment's load
                // the wave has issued the remaining fragment loads of the tile and then exactly
                // PASSES stores, so the fragment has landed once at most that many operations
                // are outstanding.  (Guarded-off K-steps only make the count stricter.)
                // Instances with run-time K guards have drained everything above.
                constexpr int kBehindAll = EXACT ? (KHM * KSM - 1 - idx) + PASSES : 0;
                constexpr int kBehind = kBehindAll < 63 ? kBehindAll : 63;
                asm volatile("s_waitcnt vmcnt(%1)" : "+v"(xf[kh][ks]) : "n"(kBehind) : "memory");
                const Vec xv = __builtin_bit_cast(Vec, xf[kh][ks]);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[nt] = TR::mfma(wf[kh][ks][nt], xv, acc[nt]);
            }
        });

        // where this tile's rows go (wave-uniform part), then move on and prefetch
        const unsigned cur_m0 = m0, cur_wo0 = wo0, cur_rowid0 = img0 * (unsigned)g.Hout + ho0;
        advance();
        // The next tile's input stays in flight across the epilogue.  After the wave's last tile
        // this fetches a tile that is never used: lanes past the end of the image get zeros from
        // the range check, the others read valid input, so the load is always safe.
        load_tile(xf);

        // ---- epilogue: round, ReLU, transpose through LDS, row-contiguous stores ----
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // four consecutive output columns of pixel r
                unsigned char *dst = slab + r * PITCH + (32 * nt + 8 * q + 4 * hf) * EB;
                if constexpr (EB == 2) {
                    u32x2 pk = {pack2<T>(acc[nt][4 * q], acc[nt][4 * q + 1]), pack2<T>(acc[nt][4 * q + 2], acc[nt][4 * q + 3])};
                    if (RELU) {
                        // max(v, 0) on the rounded 16-bit patterns as signed integers: negative
                        // values (sign bit set) become +0, everything else is unchanged
                        typedef short s16x4 __attribute__((ext_vector_type(4)));
                        const s16x4 z = {0, 0, 0, 0};
                        pk = __builtin_bit_cast(u32x2, __builtin_elementwise_max(__builtin_bit_cast(s16x4, pk), z));
                    }
                    *reinterpret_cast<u32x2 *>(dst) = pk;
                } else {
                    floatx4_t v = {acc[nt][4 * q], acc[nt][4 * q + 1], acc[nt][4 * q + 2], acc[nt][4 * q + 3]};
                    if (RELU) {
                        // the same rule on the fp32 patterns (a negative zero or a NaN with the sign bit set becomes +0)
                        typedef int s32x4 __attribute__((ext_vector_type(4)));
                        const s32x4 z = {0, 0, 0, 0};
                        v = __builtin_bit_cast(floatx4_t, __builtin_elementwise_max(__builtin_bit_cast(s32x4, v), z));
                    }
                    *reinterpret_cast<floatx4_t *>(dst) = v;
                }
            }
        wave_lds_sync();
        if (a.pace) {  // wave-uniform, scalar instructions only; the spin is bounded whatever the clock reads
            for (int spin = 0; spin < 1024 && (long long)(((unsigned long long)wall_clock64() << 8) - pace_next) < 0; ++spin)
                __builtin_amdgcn_s_sleep(1);
            pace_next += a.pace;
        }
        // Stores go through a range-checked buffer resource based at the tile's first output
        // row: lanes that have nothing to store (pixels past the end, cropped columns) use an
        // out-of-range offset and the hardware drops them.  No branch surrounds a store, so
        // the input prefetch above is not held back by store completion.
        {
            unsigned long long base_el, left_el;  // first element of the resource, elements to the end of y
            if (a.linear_out) {
                base_el = (unsigned long long)cur_m0 * (unsigned)g.NCo;
                left_el = ((unsigned long long)g.M - cur_m0) * (unsigned)g.NCo;
            } else {
                base_el = (unsigned long long)cur_rowid0 * (unsigned)g.out_row;
                left_el = (y_rows_total - cur_rowid0) * (unsigned)g.out_row;
            }
            const unsigned long long left_b = left_el * (unsigned long long)EB;
            const __amdgpu_buffer_rsrc_t yr = __builtin_amdgcn_make_buffer_rsrc(
                y + base_el, 0, (int)(left_b > 0x7fffffffull ? 0x7fffffffull : left_b), 0x00020000);
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                const u32x4 v = *reinterpret_cast<const u32x4 *>(slab + st_lds[p]);
                unsigned off;
                if (a.linear_out) {
                    off = st_lin[p];
                } else {
                    const unsigned t = cur_wo0 + (unsigned)st_row[p];
                    const unsigned q = small_div(t, a.mgW, (unsigned)g.Wf_out);
                    const unsigned oc = (t - q * (unsigned)g.Wf_out) * (unsigned)g.NCo + (unsigned)st_col[p];
                    const bool ok = st_lin[p] != kOutOfRange && cur_m0 + (unsigned)st_row[p] < (unsigned)g.M &&
                                    oc + (unsigned)EO <= (unsigned)g.out_row;
                    off = ok ? (unsigned)EB * (q * (unsigned)g.out_row + oc) : kOutOfRange;
                }
                __builtin_amdgcn_raw_buffer_store_b128(v, yr, off, 0, 2 /* nt */);
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
    // fp32 rows of 128 columns would need more LDS for the four waves' slabs than a workgroup may declare;
    // fc_stream_shape never picks those instances for fp32
    if constexpr (sizeof(T) == 4 && NT > 2) return (int)hipErrorInvalidValue; else {
    StreamArgs a;
    a.MT = (unsigned)((g.M + 31) / 32);
    a.NG = (g.NCo + 32 * NT - 1) / (32 * NT);
    a.ksteps = ksteps;
    // Persistent grid: the workgroups the launch bounds keep resident on every compute unit, rounded
    // so that the wave count is a multiple of NG (each M tile is then finished by NG waves running
    // side by side) and no more tiles in flight than there are tiles.
    FcDevice dev;
    if (int e = fc_device(&dev)) return e;
    const unsigned per_cu = (unsigned)OCC;
    const unsigned parts = a.MT >= 64 * dev.xcds ? dev.xcds : 1;  // deal tiles per XCD unless there are too few tiles to split
    const unsigned waves = dev.cus * per_cu * 4u / parts;  // per XCD
    a.deal = fc_make_deal(a.MT, parts, waves / (unsigned)a.NG, g.KH, g.Wf_out);
    const long long J = a.deal.J;
    const long long S = (long long)a.deal.stride * 32, plane = (long long)g.Hout * g.Wf_out;
    a.dI = (unsigned)(S / plane);
    a.dH = (unsigned)((S % plane) / g.Wf_out);
    a.dW = (unsigned)((S % plane) % g.Wf_out);
    a.mgW = magic_for((unsigned)g.Wf_out);
    a.mgH = magic_for((unsigned)g.Hout);
    a.x_bytes = (unsigned)((long long)g.N * g.H * g.in_row * (long long)sizeof(T));
    a.linear_out = g.out_row == g.Wf_out * g.NCo ? 1 : 0;
    a.pace = g.unpaced ? 0u : fc_store_pace(((double)g.N * g.H * g.in_row + (double)g.N * g.Hout * g.out_row) * (double)sizeof(T),
                           (a.MT + a.deal.stride - 1) / a.deal.stride, dev.wall_khz);
    const unsigned blocks = (unsigned)((J * a.NG + 3) / 4) * a.deal.parts;
    const bool exact = g.KH == KHM && ksteps == KSM;
#define FC_GO(EX, RL)                                                                       \
    conv_stream_kernel<TR, NT, KHM, KSM, OCC, EX, RL><<<blocks, 256, 0, st>>>(              \
        g, a, (const T *)x, (const typename TR::Vec *)wp, (const T *)bias, (T *)y)
    if (exact && g.relu) FC_GO(true, true);
    else if (exact) FC_GO(true, false);
    else if (g.relu) FC_GO(false, true);
    else FC_GO(false, false);
#undef FC_GO
    return (int)hipGetLastError();
    }
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
    // the operand chunk the plan packed the filter in (g.epc) picks the traits
    if (dt == FOLDCONV_F16 && g.epc == 8) return launch_shape<F16Traits>(g, sh, x, w_pack, bias, y, st);
    if (dt == FOLDCONV_BF16 && g.epc == 8) return launch_shape<BF16Traits>(g, sh, x, w_pack, bias, y, st);
    if (dt == FOLDCONV_F16 && g.epc == 4) return launch_shape<F16HalfTraits>(g, sh, x, w_pack, bias, y, st);
    if (dt == FOLDCONV_BF16 && g.epc == 4) return launch_shape<BF16HalfTraits>(g, sh, x, w_pack, bias, y, st);
    if (dt == FOLDCONV_F32 && g.epc == 4) return launch_shape<F32ChunkTraits>(g, sh, x, w_pack, bias, y, st);
    if (dt == FOLDCONV_F32 && g.epc == 2) return launch_shape<F32PairTraits>(g, sh, x, w_pack, bias, y, st);
    return (int)hipErrorInvalidValue;
}
