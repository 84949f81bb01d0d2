// Streaming MFMA convolution with a channels-first (NCHW) output (and, on request, input),
// for width- and height-folded plans of small-K layers.
//
// The filter-stationary streaming kernel gives every wave 64 output columns
// n = g*C_out + co, i.e. (part of) one output slot g.  In a channels-first
// output y[n][co][h][F*w'+g] the slots of one folded pixel are neighbours along
// w, so contiguous stores need all F slots of a run of pixels in one place.
// Here one workgroup holds every column group of an M tile (F*C_out/64 waves, at
// most 16): each wave computes its 32 pixels x 64 columns exactly as the
// streaming kernel does (filter fragments resident in registers, band walk, bias
// as a rank-1 MFMA), the workgroup assembles the 32 x F*C_out tile in LDS, and
// all threads write it out channel by channel: a thread reads the same four
// channels of eight neighbouring slots (eight 8-byte LDS reads), regroups the
// 16-bit values in registers into four 16-byte pieces, one per channel, each
// holding 8 consecutive image columns; a wave's store instruction covers a
// contiguous run of 64 such pieces of one channel row.
//
// Height-folded plans (HF: the plan describes the transposed image, its rows are image
// columns and its folded axis is the image height) take the same route with another tile
// shape.  There the contiguous axis of y, w, runs across plan rows, so an M tile is 32
// consecutive plan rows at one folded column b' (instead of 32 consecutive folded pixels of a
// row), and a thread of the write-out reads the same four channels of one slot from eight
// neighbouring pixels: again four 16-byte pieces of 8 consecutive image columns, now at image
// row h = F*b' + g.  Two such tiles, one above the other, are assembled in the two LDS buffers
// before either is written out, so that eight neighbouring lanes store 64 consecutive image
// columns of a channel row: whole 128-byte lines (half lines, written tile by tile, cost a
// quarter of the launch).
//
// HQ instances (height folds whose F*C_out is a multiple of 128 or 256) go further: a workgroup owns one of HQ = 2
// or 4 parts of the columns (the slots of that part of the fold) for its whole life and assembles 2 * HQ tiles,
// 128 or 256 plan rows, in the same LDS before writing them out, its waves forming HQ groups that compute two of
// the tiles each.  Sixteen or thirty-two neighbouring lanes then store 256 consecutive bytes, or a whole row, of a
// channel plane, and the lanes behind them the rows below it in the same plane.  A stand-alone stream of these
// store patterns over the 411 MB output of the headline layer takes 100 us with 128-byte runs, 83 us with
// 256-byte runs or whole rows, 78 us with the rows of one channel next to each other in a wave (68 us with the
// 1 KB runs of the width fold): the store pattern is what bounds this kernel.
//
// XN instances (height folds) read a channels-first input as well: the folded pixel's channel f*C_in + c of
// plan row a is x[n][c][F*b'+f][a], so a lane's fragment of eight K-contiguous values is gathered with eight
// 2-byte loads (one register each, paired up after they land: on this GPU a 16-bit load into one half of a
// register clears the other half).  The 32 pixels of a tile are consecutive plan rows a, so the lanes of a
// load read 64 consecutive bytes of one image row; the separate fold pass and its round trip through memory
// fall away (paper: Eq. "width_fold_def", along h, applied in the load addressing).  For a width fold the
// same gather would have the lanes F elements apart (x[n][c][a][F*b'+f], b' across the lanes): measured
// three times slower than the fold pass it replaces.  Width folds therefore stage the channels-first rows
// through LDS instead (XW instances): per tile every thread fetches one 16-byte piece of a channel row (eight
// consecutive image columns of the few input rows the tile's pixels need) and scatters it, 2 bytes at a time,
// to where those values sit in the folded rows x'[n][h][w*C + c]; the waves then read their fragments from that
// copy with 16-byte LDS reads.  Two such stage buffers alternate, so the trip keeps its single barrier; the
// piece of the tile after next stays in flight across the write-out like the fragments it replaces.
// paper: Eq. "new_conv_H", Eq. "bias_construct"; the Reconstruct step
// w = F w' + f (h = F h' + f for a height fold), applied on the way to a channels-first tensor.
#include <hip/hip_runtime.h>
#include <type_traits>

#include "launch.h"
#include "lds_attr.h"
#include "mfma_types.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <typename TR>
__device__ __forceinline__ unsigned pack2n(float a, float b);
template <>
__device__ __forceinline__ unsigned pack2n<F16Traits>(float a, float b) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 v = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(unsigned, v);
}
template <>
__device__ __forceinline__ unsigned pack2n<BF16Traits>(float a, float b) {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    b2 v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(unsigned, v);
}

constexpr unsigned kOutOfRangeN = 0xfffffff0u;  // beyond any resource extent used here (extents stay below 2^32 - 64)

struct NchwArgs {
    unsigned MT;          // 32-pixel M tiles (HF: pairs of them, 64 plan rows of one folded column)
    FcDeal deal;          // how M tiles are dealt to the XCDs: deal.J workgroups per XCD, one tile each at a time
    unsigned dW, dH, dI;  // the stride of a workgroup's tile walk, 32*deal.stride pixels, as (folded column, row, image) steps
    unsigned mgW, mgH;    // ceil(2^32 / Wf_out), ceil(2^32 / Hout)
    unsigned x_bytes, y_bytes;
    int ksteps;           // 16-wide K-steps per kh actually walked (<= KSM)
    int pitch;            // bytes per pixel row of the assembled tile
    int skew;             // extra bytes in front of every further group of 8 slots (LDS bank spread)
    unsigned tiles_ab;    // HF: tile pairs per folded column, ceil(Hout / 64)
    unsigned pace;        // wall-clock ticks * 256 between a workgroup's store bursts, 0 = unpaced (fc_store_pace)
    // XN, XW: element strides of the channels-first input: one channel plane, one step along the plan's rows,
    // one step along the plan's (unfolded) columns
    unsigned xP, xsA, xsB;
    // XW: the stage of folded input rows in LDS: rows per buffer, bytes per row (zero halo, the row, zero halo),
    // elements of the halo in front, 16-byte pieces per channel row of the image
    int stage_rows, stage_pitch, halo_l, xW8;
};

template <int I, int N, class F>
__device__ __forceinline__ void static_for_n(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for_n<I + 1, N>(f);
    }
}

// floor(t / d) for t < d + 64 and d < 65000, with mg = ceil(2^32 / d)
__device__ __forceinline__ unsigned small_div_n(unsigned t, unsigned mg, unsigned d) {
    return d == 1u ? t : __umulhi(t, mg);
}

// EXACT: g.KH == KHM and a.ksteps == KSM, so the K loops carry no run-time guards.
// HQ: 0, or the number of parts the columns are divided into (2 or 4; one workgroup each, 2 * HQ tiles per block of rows)
template <typename TR, int KHM, int KSM, bool EXACT, bool RELU, bool HF, bool XN, int HQ, bool XW>
__global__ void __launch_bounds__(1024, 1)
conv_stream_nchw_kernel(ConvGeom g, NchwArgs a, const typename TR::T *__restrict__ x, const u32x4 *__restrict__ wp,
                        const typename TR::T *__restrict__ bias, typename TR::T *__restrict__ y) {
    using T = typename TR::T;
    using Vec = typename TR::Vec;
    constexpr int NT = 2, COLS = 64;
    static_assert(HF || !HQ, "quads are a height-fold layout");
    static_assert(!XW || (!HF && !XN), "the staged input read is the width fold's");
    extern __shared__ __attribute__((aligned(16))) unsigned char tile_lds[];  // two (HQ: four) tiles of 32 * pitch bytes

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int r = lane & 31, hf = lane >> 5;
    // Workgroup b runs on XCD b % parts; M tiles follow the workgroups in chunks (FcDeal).  HQ: two workgroups on
    // the same XCD, one per half of the columns, walk the same quads.
    const unsigned xcd = blockIdx.x % a.deal.parts, wg = blockIdx.x / a.deal.parts;
    constexpr int QP = HQ ? HQ : 1;
    static_assert(HQ == 0 || HQ == 2 || HQ == 4, "pairs, or the columns in two or four parts");
    const int col_half = HQ ? (int)(wg % (unsigned)QP) : 0;
    const int col0 = col_half * (g.NCo / QP);            // first column the workgroup's LDS tiles hold
    const int wpg = HQ ? (int)(blockDim.x / (64 * QP)) : 1;  // HQ: waves per tile group = (F*C_out / QP) / 64
    const int tg = HQ ? wave / wpg : 0;                  // HQ: the wave computes tiles 2*tg and 2*tg + 1 of a quad
    const int n_lo = HQ ? col0 + (wave - tg * wpg) * COLS : wave * COLS;
    const int KH = EXACT ? KHM : g.KH, KS = EXACT ? KSM : a.ksteps;

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
                if (kh < KH && ks < KS && e < e_hi) {
                    const int q = (e - g.e_min) >> 3;
                    const long long ci = g.compact ? fc_compact_chunk<8>(g, kh, q, n)
                                                   : ((long long)kh * q_per_kh + q) * g.NCo + n;
                    if (ci >= 0) v = wp[ci];  // off-band chunks of the compact form are zeros
                }
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
        if (g.has_bias && hf == 0) bf[nt][0] = bias[n % g.Co];
    }
    unsigned ksmask = 0;  // K-steps whose chunk lies inside this wave's band window
#pragma unroll
    for (int ks = 0; ks < KSM; ++ks)
        if (ks < KS && e0 + 16 * ks < e_hi) ksmask |= 1u << ks;

    // Range-checked resources: a lane with nothing to read (zero padding, pixels past the end)
    // or nothing to store uses an out-of-range offset; reads return zeros, stores are dropped.
    // The input loads are issued from inline assembly and waited for with explicit counts (see
    // the loop head): the compiler's own wait insertion would make every wave wait for its
    // previous tile's stores before touching the next tile's input.
    u32x4 xr;
    {
        const unsigned long long xa = (unsigned long long)x;
        xr[0] = __builtin_amdgcn_readfirstlane((unsigned)xa);
        xr[1] = __builtin_amdgcn_readfirstlane((unsigned)(xa >> 32) & 0xffffu);  // stride 0: raw buffer, byte offsets
        xr[2] = __builtin_amdgcn_readfirstlane(a.x_bytes);
        xr[3] = __builtin_amdgcn_readfirstlane(0x00020000u);
    }
    const __amdgpu_buffer_rsrc_t yr = __builtin_amdgcn_make_buffer_rsrc(y, 0, (int)a.y_bytes, 0x00020000);

    // ---- this thread's share of the write-out.  W fold: pixel sp of the tile, slots [8*sg8, 8*sg8+8),
    //      channels [4*co4, 4*co4+4): 32 * (F/8) threads per channel quadruple, C_out/4 quadruples.
    //      HF: pixels [8*da8, 8*da8+8) of the tile pair (da8 < 4: first tile, else second), slots hg and
    //      hg + F/2 in turn, channels [4*co4, 4*co4+4); da8 runs fastest over the lanes, so eight lanes
    //      store 128 consecutive bytes of a channel row.  HQ: da8 < 16 over the four tiles of the quad (sixteen
    //      lanes store 256 consecutive bytes), slots hg and hg + F/4 of the workgroup's half of the fold.
    const int g8n = HF ? 1 : g.F >> 3;
    const int per_c4 = 32 * g8n;
    const int c4n = g.Co >> 2;
    constexpr int DAB = HQ ? (QP == 2 ? 4 : 5) : 3;  // log2 of the 8-pixel groups along the plan rows of a pair or quad
    const int slot_step = HQ ? g.F / (2 * QP) : g.F >> 1;   // HF: the thread's second slot lies this far from its first
    // (HQ: the lanes run over the rows of one channel quadruple before they go on to the next: a wave's store covers
    // neighbouring rows of one channel plane, 74 us on the headline layer against 85 us with the channels next)
    const int co4 = HF ? (HQ ? t / ((1 << DAB) * slot_step) : (t >> DAB) % c4n) : t / per_c4;
    const int sp = HF ? 0 : (t - co4 * per_c4) / g8n;
    const int sg8 = HF ? 0 : (t - co4 * per_c4) - sp * g8n;
    const int da8 = HF ? t & ((1 << DAB) - 1) : 0;
    const int hg = HF ? (HQ ? (t >> DAB) % slot_step : t / ((1 << DAB) * c4n)) : 0;  // below slot_step: the block has F*C_out threads
    // W fold: + k * C_out * 2 per slot; HF: + k * pitch per pixel, + slot_step * C_out * 2 for the second slot
    const int rd_off = HF ? ((da8 >> 2) * 32 + 8 * (da8 & 3)) * a.pitch + (hg * g.Co + 4 * co4) * 2
                          : sp * a.pitch + (8 * sg8 * g.Co + 4 * co4) * 2 + sg8 * a.skew;
    const int rd_step = HF ? a.pitch : g.Co * 2;
    // bytes per channel plane: image H_out x W_out (W fold: Hout x out_row; HF: out_row x Hout, the plan is transposed)
    const unsigned plane_b = 2u * (unsigned)g.Hout * (unsigned)g.out_row;

    const unsigned t_first = fc_deal_first_tile(a.deal, xcd, HQ ? wg / (unsigned)QP : wg);  // the workgroup's first tile

    // The workgroup's current tile.  W fold: 32 consecutive folded pixels from m0 = (img0, ho0, wo0), advanced
    // incrementally.  HF: tile pair `tile` = (img0 * tiles_ab + pair) * Wf_out + wo0 (folded column fastest:
    // consecutive pairs share their 64 input rows); its half `sub` holds plan rows [ho0, ho0 + 32),
    // ho0 = 64 * pair + 32 * sub.  A half that starts at or beyond Hout reads zeros and stores nothing.
    // HQ: the same with quads of 128 plan rows; the wave's tiles are 2*tg + sub: ho0 = 128 * quad + 32 * (2*tg + sub).
    unsigned m0 = t_first * 32u;
    unsigned wo0, ho0, img0;
    unsigned row0 = 0;  // HF: first plan row of the pair or quad
    unsigned cur_tile = t_first;
    auto place = [&](unsigned tile, unsigned sub) {
        if (HF) {
            cur_tile = tile;
            // past the last pair the position is never used for a store; keep it inside the tensor for the prefetch
            const unsigned tl = tile < a.MT ? tile : a.MT - 1u;
            const unsigned rb = tl / (unsigned)g.Wf_out;  // (image, pair)
            wo0 = tl - rb * (unsigned)g.Wf_out;
            img0 = rb / a.tiles_ab;
            row0 = (rb - img0 * a.tiles_ab) * (unsigned)(64 * QP);
            ho0 = row0 + 32u * (HQ ? 2u * (unsigned)tg + sub : sub);
        } else {
            wo0 = m0 % (unsigned)g.Wf_out;
            const unsigned rowid = m0 / (unsigned)g.Wf_out;
            ho0 = rowid % (unsigned)g.Hout;
            img0 = rowid / (unsigned)g.Hout;
        }
    };
    place(t_first, 0);
    // pixel i of the tile at (wo_base, ho_base, img_base): its coordinates, and whether it exists
    auto pixel = [&](unsigned wo_base, unsigned ho_base, unsigned img_base, unsigned i, unsigned &wo, unsigned &ho,
                     unsigned &img) {
        if (HF) {
            wo = wo_base;
            ho = ho_base + i;
            img = img_base;
            return;
        }
        const unsigned tt = wo_base + i;
        const unsigned q = small_div_n(tt, a.mgW, (unsigned)g.Wf_out);
        wo = tt - q * (unsigned)g.Wf_out;
        const unsigned hr = ho_base + q;
        const unsigned q2 = small_div_n(hr, a.mgH, (unsigned)g.Hout);
        ho = hr - q2 * (unsigned)g.Hout;
        img = img_base + q2;
    };
    auto advance = [&]() {  // W fold only
        m0 += a.deal.stride * 32u;
        wo0 += a.dW;
        unsigned c = wo0 >= (unsigned)g.Wf_out ? 1u : 0u;
        wo0 -= c * (unsigned)g.Wf_out;
        ho0 += a.dH + c;
        c = ho0 >= (unsigned)g.Hout ? 1u : 0u;
        ho0 -= c * (unsigned)g.Hout;
        img0 += a.dI + c;
    };

    // XN: where the K value e_lo + 8*h + 16*ks + i (h = 0, 1: the two halves of the wave) sits relative to plan
    // row 0, unfolded column F*b' of its image: channel plane and unfolded column (the value's folded channel
    // k = f*C + c lies dw = floor(k / C) columns on).  Wave-uniform, so the table lives in scalar registers:
    // entry [ks][i] for h = 0 and what h = 1 adds to it.
    int goff[XN ? KSM : 1][XN ? 8 : 1], goff_hi[XN ? KSM : 1][XN ? 8 : 1];
    if constexpr (XN) {
#pragma unroll
        for (int ks = 0; ks < KSM; ++ks)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                int at[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int k = e_lo + 8 * h + 16 * ks + i;
                    int dw = k / g.C;
                    if (k - dw * g.C < 0) --dw;
                    at[h] = (k - dw * g.C) * (int)a.xP + dw * (int)a.xsB;
                }
                goff[ks][i] = at[0];
                goff_hi[ks][i] = at[1] - at[0];
            }
    }
    // An input fragment: one 16-byte load, or (XN) eight zero-extended 2-byte loads.
    struct Halves { unsigned d[8]; };
    using Frag = std::conditional_t<XN, Halves, u32x4>;
    Frag xf[KHM][KSM];
    constexpr int LPF = XN ? 8 : 1;  // hand-issued loads per fragment
    auto load_tile = [&]() {
        unsigned wo, ho, img;
        pixel(wo0, ho0, img0, (unsigned)r, wo, ho, img);
        const bool vm = HF ? (cur_tile < a.MT && ho < (unsigned)g.Hout) : m0 + (unsigned)r < (unsigned)g.M;
        const int col0 = (int)wo * g.FC + e0;  // column of K-step 0 inside the input row
        const int pix0 = ((int)(img * (unsigned)g.H + ho) - g.pad_h) * g.in_row + col0;
        // XN: element offset of (plan row ho - pad_h, unfolded column F*wo, channel 0) of image img
        const int nc0 = (int)(img * (unsigned)g.C) * (int)a.xP + ((int)ho - g.pad_h) * (int)a.xsA + (int)wo * g.F * (int)a.xsB;
        // the lane's half of the wave, re-read here so that the per-lane form of the table is not kept in
        // vector registers across the loop
        int half = hf;
        if constexpr (XN) asm volatile("" : "+v"(half));
#pragma unroll
        for (int kh = 0; kh < KHM; ++kh) {
            const int hi = (int)ho + kh - g.pad_h;
            const bool rv = vm && kh < KH && hi >= 0 && hi < g.H;
#pragma unroll
            for (int ks = 0; ks < KSM; ++ks) {
                // in range: row hi exists and the 8-element chunk [col, col+8) lies inside it (chunks do not
                // straddle the ends of a row: its length and col are multiples of 8)
                const int col = col0 + 16 * ks;
                const bool ok = rv && ((ksmask >> ks) & 1u) && col >= 0 && col < g.in_row;
                if constexpr (XN) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const unsigned voff = ok ? 2u * (unsigned)(nc0 + kh * (int)a.xsA + goff[ks][i] + half * goff_hi[ks][i]) : kOutOfRangeN;
                        asm volatile("buffer_load_ushort %0, %1, %2, 0 offen" : "=v"(xf[kh][ks].d[i]) : "v"(voff), "s"(xr) : "memory");
                    }
                } else {
                    const unsigned voff = ok ? 2u * (unsigned)(pix0 + kh * g.in_row + 16 * ks) : kOutOfRangeN;
                    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(xf[kh][ks]) : "v"(voff), "s"(xr) : "memory");
                }
            }
        }
    };

    // Nothing the compiler tracks may be in flight when the hand-counted loads start.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if constexpr (!XW) load_tile();
    // Drain the first tile's loads here: the loop head then only ever waits for loads that were
    // issued ahead of the stores of the previous tile, and leaves those stores in flight.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // Store pacing (fc_store_pace): the wave's next store burst is not issued before this time (ticks * 256).
    // The workgroups start a fraction of an interval apart, so that their bursts do not all fall together.
    unsigned long long pace_next =
        a.pace ? ((unsigned long long)wall_clock64() << 8) + (unsigned long long)a.pace * blockIdx.x / gridDim.x : 0ull;
    auto pace = [&]() {
        if (a.pace) {  // wave-uniform, scalar instructions only; the spin is bounded whatever the clock reads
            for (int spin = 0; spin < 1024 && (long long)(((unsigned long long)wall_clock64() << 8) - pace_next) < 0; ++spin)
                __builtin_amdgcn_s_sleep(1);
            pace_next += a.pace;
        }
    };

    // Waits until at most N vector-memory operations are outstanding, and ties the fragment's registers to the wait.
    auto wait_frag = [&](Frag &f, auto n) {
        constexpr int N = decltype(n)::value;
        if constexpr (XN)
            asm volatile("s_waitcnt vmcnt(%8)"
                         : "+v"(f.d[0]), "+v"(f.d[1]), "+v"(f.d[2]), "+v"(f.d[3]), "+v"(f.d[4]), "+v"(f.d[5]), "+v"(f.d[6]), "+v"(f.d[7])
                         : "n"(N) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(%1)" : "+v"(f) : "n"(N) : "memory");
    };
    auto frag_vec = [&](const Frag &f) {
        if constexpr (XN) {
            const u32x4 v = {f.d[0] | (f.d[1] << 16), f.d[2] | (f.d[3] << 16), f.d[4] | (f.d[5] << 16), f.d[6] | (f.d[7] << 16)};
            return __builtin_bit_cast(Vec, v);
        } else {
            return __builtin_bit_cast(Vec, f);
        }
    };
    // The fragments in xf times the resident filter, bias included.  STORES_BEHIND: the stores the wave issued
    // after the loads of xf.
    auto multiply = [&](floatx16_t (&acc)[NT], auto stores_behind) {
        constexpr int STORES_BEHIND = decltype(stores_behind)::value;
        floatx16_t zero;
#pragma unroll
        for (int i = 0; i < 16; ++i) zero[i] = 0.0f;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = TR::mfma(bf[nt], ones, zero);
        if (!EXACT && !XW) {
            // Instances with run-time K guards drain every fragment load here, ahead of the guards:
            // a fragment whose K-step is guarded off is never waited for below, and its registers
            // must not be handed to anything else while its load is still in flight.
#pragma unroll
            for (int i = 0; i < KHM * KSM; ++i) wait_frag(xf[i / KSM][i % KSM], std::integral_constant<int, 0>{});
        }
        static_for_n<0, KHM * KSM>([&](auto step) {
            constexpr int idx = decltype(step)::value;
            constexpr int kh = idx / KSM, ks = idx % KSM;
            if (EXACT || (kh < KH && ks < KS)) {
                // Vector-memory operations retire in issue order.  Behind this fragment's load the
                // wave has issued the remaining fragment loads of the tile and then exactly
                // STORES_BEHIND stores, so the fragment has landed once at most that many operations
                // are outstanding.  Instances with run-time K guards have drained everything above.
                constexpr int kBehind = EXACT ? (KHM * KSM - 1 - idx) * LPF + STORES_BEHIND : 0;
                if constexpr (!XW) wait_frag(xf[kh][ks], std::integral_constant<int, kBehind>{});  // XW: read from LDS
                const Vec xv = frag_vec(xf[kh][ks]);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[nt] = TR::mfma(wf[kh][ks][nt], xv, acc[nt]);
            }
        });
    };
    // Round (and clamp) the wave's 32 x 64 results into pixel rows of F*C_out columns at tb.
    auto assemble = [&](const floatx16_t (&acc)[NT], unsigned char *tb) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                u32x2 pk = {pack2n<TR>(acc[nt][4 * q], acc[nt][4 * q + 1]), pack2n<TR>(acc[nt][4 * q + 2], acc[nt][4 * q + 3])};
                if (RELU) {
                    // max(v, 0) on the rounded 16-bit patterns as signed integers
                    typedef short s16x4 __attribute__((ext_vector_type(4)));
                    const s16x4 z = {0, 0, 0, 0};
                    pk = __builtin_bit_cast(u32x2, __builtin_elementwise_max(__builtin_bit_cast(s16x4, pk), z));
                }
                const int n = n_lo + 32 * nt + 8 * q + 4 * hf;
                const int slot8 = (n / g.Co) >> 3;
                *reinterpret_cast<u32x2 *>(tb + r * a.pitch + (n - col0) * 2 + slot8 * a.skew) = pk;
            }
    };
    // Eight 8-byte reads at src (four channels of eight neighbouring slots or pixels), regrouped into four
    // 16-byte pieces of eight consecutive image columns, one per channel plane from off0 on.
    auto write_out = [&](const unsigned char *src, unsigned off0, bool ok) {
        u32x2 v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = *reinterpret_cast<const u32x2 *>(src + k * rd_step);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            u32x4 out;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const unsigned lo = v[2 * j][i >> 1], hi = v[2 * j + 1][i >> 1];
                out[j] = (i & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
            }
            __builtin_amdgcn_raw_buffer_store_b128(out, yr, ok ? off0 + (unsigned)i * plane_b : kOutOfRangeN, 0, 2 /* nt */);
        }
    };

    if constexpr (HF) {
        // Per tile pair: both halves multiplied and assembled (one LDS buffer each), one barrier, eight stores
        // per thread, and a second barrier before the next pair's first half overwrites buffer 0.  The input
        // of the half after the current one is always in flight: behind the loads of a first half lie the
        // eight stores of the pair before it, behind those of a second half none.
        unsigned char *const tb0 = tile_lds + (HQ ? 2 * tg : 0) * (32 * a.pitch), *const tb1 = tb0 + 32 * a.pitch;
        for (unsigned mt = t_first; mt < a.MT; mt += a.deal.stride) {
            floatx16_t acc[NT];
            multiply(acc, std::integral_constant<int, 8>{});
            const unsigned cur_wo0 = wo0, cur_ho0 = row0, cur_img0 = img0;  // first plan row of the pair or quad
            place(mt, 1);
            load_tile();
            __syncthreads();  // every wave has finished reading the previous pair out of both buffers
            assemble(acc, tb0);
            multiply(acc, std::integral_constant<int, 0>{});
            // After the workgroup's last pair this fetches a tile that is never used; every lane's address is
            // either inside x or out of the resource's range, so the load is always safe.
            place(mt + a.deal.stride, 0);
            load_tile();
            assemble(acc, tb1);
            __syncthreads();
            pace();
            // ---- write out y[img][4*co4+i][F*wo + hg (+ F/2)][ho0 + 8*da8 .. +8) for i = 0..3 ----
            const unsigned w0 = cur_ho0 + 8u * (unsigned)da8;  // first image column of the piece
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const unsigned slot = (unsigned)(col_half * (g.F / QP) + hg + half * slot_step);
                const unsigned h = cur_wo0 * (unsigned)g.F + slot;  // image row
                const bool ok = h < (unsigned)g.out_row && w0 < (unsigned)g.Hout;  // Hout % 8 == 0: a piece is whole or absent
                const unsigned off0 =
                    2u * (((cur_img0 * (unsigned)g.Co + 4u * (unsigned)co4) * (unsigned)g.out_row + h) * (unsigned)g.Hout + w0);
                write_out(tile_lds + rd_off + half * (slot_step * g.Co * 2), off0, ok);
            }
        }
    } else if constexpr (XW) {
        // ---- width fold, channels-first input staged through LDS ----------------------------------------
        // No tile crosses an image here (the host checks that an image is a whole number of tiles), so a
        // tile's pixels lie in output rows ho0 .. ho0 + R - 1 of one image and need the input rows
        // ho0 - pad_h + s, s < stage_rows: stage row s.  Pixel (ho0 + q, wo) reads its fragment for kh from
        // stage row q + kh at folded column wo*F*C + e; the zero halos at both ends of a stage row and the
        // zeros that out-of-range loads return are the zero padding.
        unsigned char *const stage0 = tile_lds + 2 * 32 * a.pitch;
        const int stage_bytes = a.stage_rows * a.stage_pitch;
        for (int o = t * 16; o < 2 * stage_bytes; o += (int)blockDim.x * 16)
            *reinterpret_cast<u32x4 *>(stage0 + o) = u32x4{0u, 0u, 0u, 0u};  // the halos stay zero from here on
        // this thread's piece of a stage buffer: stage row ps, channel pc, image columns [8*pw8, 8*pw8 + 8)
        const int per_row = g.C * a.xW8;
        const int ps = t / per_row, pc = (t - ps * per_row) / a.xW8, pw8 = t - ps * per_row - pc * a.xW8;
        const bool p_has = ps < a.stage_rows;
        const int p_lds = ps * a.stage_pitch + (a.halo_l + 8 * pw8 * g.C + pc) * 2;  // + i * C * 2 for column 8*pw8 + i
        const int p_x = pc * (int)a.xP + 8 * pw8;                                    // + image and row
        struct Pos { unsigned m0, wo0, ho0, img0; };
        auto next_pos = [&](Pos &p) {
            p.m0 += a.deal.stride * 32u;
            p.wo0 += a.dW;
            unsigned c = p.wo0 >= (unsigned)g.Wf_out ? 1u : 0u;
            p.wo0 -= c * (unsigned)g.Wf_out;
            p.ho0 += a.dH + c;
            c = p.ho0 >= (unsigned)g.Hout ? 1u : 0u;
            p.ho0 -= c * (unsigned)g.Hout;
            p.img0 += a.dI + c;
        };
        u32x4 piece;
        auto piece_load = [&](const Pos &p) {
            const int hi = (int)p.ho0 - g.pad_h + ps;
            const bool ok = p_has && p.m0 < (unsigned)g.M && hi >= 0 && hi < g.H;
            const unsigned voff =
                ok ? 2u * (unsigned)((int)(p.img0 * (unsigned)g.C) * (int)a.xP + hi * (int)a.xsA + p_x) : kOutOfRangeN;
            asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(piece) : "v"(voff), "s"(xr) : "memory");
        };
        auto piece_store = [&](unsigned char *stage) {
            if (p_has) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    *reinterpret_cast<unsigned short *>(stage + p_lds + i * g.C * 2) = (unsigned short)(piece[i >> 1] >> (16 * (i & 1)));
            }
        };
        auto read_frags = [&](const unsigned char *stage, const Pos &p) {
            const unsigned tt = p.wo0 + (unsigned)r;
            const unsigned q = small_div_n(tt, a.mgW, (unsigned)g.Wf_out);
            const unsigned wo = tt - q * (unsigned)g.Wf_out;
            const int at = (int)q * a.stage_pitch + (a.halo_l + (int)wo * g.FC + e0) * 2;
#pragma unroll
            for (int kh = 0; kh < KHM; ++kh)
#pragma unroll
                for (int ks = 0; ks < KSM; ++ks) {
                    // K-steps outside the wave's band window multiply zero filter fragments: give them zeros as the
                    // global path does, whatever the input holds there
                    // (such a lane reads offset 0: the address it would form may lie past the stage)
                    const bool use = kh < KH && ((ksmask >> ks) & 1u);
                    const u32x4 v = *reinterpret_cast<const u32x4 *>(stage + (use ? at + kh * a.stage_pitch + 32 * ks : 0));
                    xf[kh][ks] = use ? v : u32x4{0u, 0u, 0u, 0u};
                }
        };
        Pos A = {m0, wo0, ho0, img0}, B = A;
        next_pos(B);
        Pos C = B;
        next_pos(C);
        __syncthreads();  // the stage buffers are zero
        piece_load(A);
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(piece) : : "memory");
        piece_store(stage0);
        piece_load(B);
        // Four stores that the range check drops, so that from the first trip on exactly four stores lie behind the
        // piece in flight when the loop waits for it.
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_raw_buffer_store_b128(u32x4{0u, 0u, 0u, 0u}, yr, kOutOfRangeN, 0, 2 /* nt */);
        __syncthreads();
        read_frags(stage0, A);
        int buf = 0;
        for (unsigned mt = t_first; mt < a.MT; mt += a.deal.stride) {
            floatx16_t acc[NT];
            multiply(acc, std::integral_constant<int, 4>{});
            // the next tile's piece has landed: behind its load lie the four stores of the tile before this one
            asm volatile("s_waitcnt vmcnt(4)" : "+v"(piece) : : "memory");
            unsigned char *const stage_next = stage0 + (buf ^ 1) * stage_bytes;
            piece_store(stage_next);
            unsigned char *tb = tile_lds + buf * (32 * a.pitch);
            assemble(acc, tb);
            // One barrier per tile: behind it the tile is assembled and the next tile's rows are staged.  Either
            // buffer is written again two tiles on, after the barrier of the tile between, which every wave passes
            // only after its reads of that buffer.
            __syncthreads();
            piece_load(C);  // the tile after next; past the end every lane's offset is out of range
            pace();
            // ---- write out y[img][4*co4+i][ho][F*wo + 8*sg8 .. +8) for i = 0..3 ----
            unsigned wo, ho, img;
            pixel(A.wo0, A.ho0, A.img0, (unsigned)sp, wo, ho, img);
            const bool ok = A.m0 + (unsigned)sp < (unsigned)g.M;
            const unsigned off0 = 2u * (((img * (unsigned)g.Co + 4u * (unsigned)co4) * (unsigned)g.Hout + ho) * (unsigned)g.out_row +
                                        wo * (unsigned)g.F + 8u * (unsigned)sg8);
            write_out(tb + rd_off, off0, ok);
            read_frags(stage_next, B);
            A = B;
            B = C;
            next_pos(C);
            buf ^= 1;
        }
    } else {
        int buf = 0;
        for (unsigned mt = t_first; mt < a.MT; mt += a.deal.stride) {
            floatx16_t acc[NT];
            multiply(acc, std::integral_constant<int, 4>{});
            const unsigned cur_m0 = m0, cur_wo0 = wo0, cur_ho0 = ho0, cur_img0 = img0;
            advance();
            // The next tile's input stays in flight across the write-out.  After the last tile this
            // fetches a tile that is never used; every lane's address is either inside x or out of
            // the resource's range, so the load is always safe.
            load_tile();
            unsigned char *tb = tile_lds + buf * (32 * a.pitch);
            assemble(acc, tb);
            // One barrier per tile is enough with two buffers: this buffer is written again two tiles
            // on, and no wave gets there before every wave has passed the next tile's barrier, which
            // each does only after finishing its reads below.
            __syncthreads();
            pace();
            // ---- write out y[img][4*co4+i][ho][F*wo + 8*sg8 .. +8) for i = 0..3 ----
            unsigned wo, ho, img;
            pixel(cur_wo0, cur_ho0, cur_img0, (unsigned)sp, wo, ho, img);
            const bool ok = cur_m0 + (unsigned)sp < (unsigned)g.M;
            const unsigned off0 = 2u * (((img * (unsigned)g.Co + 4u * (unsigned)co4) * (unsigned)g.Hout + ho) * (unsigned)g.out_row +
                                        wo * (unsigned)g.F + 8u * (unsigned)sg8);
            write_out(tb + rd_off, off0, ok);
            buf ^= 1;
        }
    }
}

static unsigned magic_for(unsigned d) { return d <= 1 ? 0u : (unsigned)(((1ULL << 32) + d - 1) / d); }

template <typename TR, int KHM, int KSM, bool HF, bool XN, int HQ, bool XW>
int launch_inst(const ConvGeom &g, int ksteps, const void *x, const void *wp, const void *bias, void *y, hipStream_t st) {
    using T = typename TR::T;
    NchwArgs a;
    NchwStage stage = {0, 0, 0, 0};
    if (XW && !fc_stream_nchw_stage(g, &stage)) return (int)hipErrorInvalidValue;
    a.stage_rows = stage.rows;
    a.stage_pitch = stage.pitch;
    a.halo_l = stage.halo_l;
    a.xW8 = g.Wf * g.F / 8;
    if (XW) {
        // no skew here: the stage buffers need its 16 KB (fc_stream_nchw_stage sized them for this pitch)
        a.skew = 0;
        a.pitch = g.NCo * 2 + 8;
    } else if (HF) {
        // a thread of the write-out reads pixels 8 rows apart and eight neighbouring lanes read pixels 8k .. 8k+7
        // of the pair: with a pitch of 8 bytes (mod 32) the lanes of a wave spread over all banks in both phases
        a.skew = 0;
        a.pitch = (HQ ? g.NCo / HQ : g.NCo) * 2 + 8;  // HQ: a workgroup's tiles hold its part of the columns
    } else {
        const int g8n = g.F / 8;
        a.skew = g8n > 1 ? 256 / g8n : 0;
        if (a.skew % 8 != 0) a.skew = 8;
        a.pitch = g.NCo * 2 + g8n * a.skew + 8;
    }
    const unsigned lds_bytes = (HQ ? 2u * HQ : 2u) * 32u * (unsigned)a.pitch + 2u * (unsigned)(stage.rows * stage.pitch);
    const unsigned threads = (unsigned)g.NCo;  // one wave per 64 columns
    // workgroups resident per compute unit: 16 waves at the register budget of the launch bounds, 160 KB of LDS
    unsigned per_cu = 1024u / threads;
    if (per_cu > 163840u / lds_bytes) per_cu = 163840u / lds_bytes;
    if (per_cu < 1) per_cu = 1;
    a.tiles_ab = HQ ? (unsigned)((g.Hout + 64 * HQ - 1) / (64 * HQ)) : (unsigned)((g.Hout + 63) / 64);
    a.MT = HF ? (unsigned)((long long)g.N * a.tiles_ab * g.Wf_out) : (unsigned)((g.M + 31) / 32);
    FcDevice dev;
    if (int e = fc_device(&dev)) return e;
    // HF: the Wf_out tiles of a row block share all their input rows; keep them in one chunk (one L2)
    // HQ: two workgroups (the two halves of the columns) walk the same quads: half as many walkers
    a.deal = fc_make_deal(a.MT, dev.xcds, dev.cus / dev.xcds * per_cu / (HQ ? (unsigned)HQ : 1u), g.KH, HF ? 8 * g.Wf_out : g.Wf_out);
    const long long S = 32LL * a.deal.stride, plane = (long long)g.Hout * g.Wf_out;
    a.dI = (unsigned)(S / plane);
    a.dH = (unsigned)((S % plane) / g.Wf_out);
    a.dW = (unsigned)((S % plane) % g.Wf_out);
    a.mgW = magic_for((unsigned)g.Wf_out);
    a.mgH = magic_for((unsigned)g.Hout);
    a.x_bytes = (unsigned)((long long)g.N * g.H * g.in_row * (long long)sizeof(T));
    a.y_bytes = (unsigned)((long long)g.N * g.Co * g.Hout * g.out_row * (long long)sizeof(T));
    a.ksteps = ksteps;
    {
        // the channels-first image: C planes of (plan rows x unfolded plan columns), transposed for a height fold
        const long long rows = g.H, cols = (long long)g.Wf * g.F;
        a.xP = (unsigned)(rows * cols);
        a.xsA = HF ? 1u : (unsigned)cols;
        a.xsB = HF ? (unsigned)rows : 1u;
    }
    // One workgroup per compute unit walks its tiles one after the other (load, multiply, assemble, barrier, write
    // out): it cannot keep the schedule the channels-last kernel keeps, and a workgroup that is behind never sleeps.
    // Offered at 6.8 TB/s it stays on schedule (measured on the headline layer: 79 us unpaced and at 7.35 TB/s,
    // 69-73 us at 6.6-7.0 TB/s), provided its input is in the caches when it starts: after a fold pass that wrote
    // x' non-temporally the launch took 81 us whatever the rate, which is why that pass writes with plain stores.
    a.pace = g.unpaced ? 0u
                       : fc_store_pace((double)a.x_bytes + (double)a.y_bytes, (a.MT + a.deal.stride - 1) / a.deal.stride,
                                       dev.wall_khz, 6.8e12);
    const unsigned blocks = a.deal.J * a.deal.parts * (HQ ? (unsigned)HQ : 1u);
    const bool exact = g.KH == KHM && ksteps == KSM;
#define FC_GO(EX, RL)                                                                                        \
    do {                                                                                                     \
        if (int e = fc_allow_full_lds<conv_stream_nchw_kernel<TR, KHM, KSM, EX, RL, HF, XN, HQ, XW>>()) return e; \
        conv_stream_nchw_kernel<TR, KHM, KSM, EX, RL, HF, XN, HQ, XW><<<blocks, threads, lds_bytes, st>>>(       \
            g, a, (const T *)x, (const u32x4 *)wp, (const T *)bias, (T *)y);                                 \
    } while (0)
    if (exact && g.relu) FC_GO(true, true);
    else if (exact) FC_GO(true, false);
    else if (g.relu) FC_GO(false, true);
    else FC_GO(false, false);
#undef FC_GO
    return (int)hipGetLastError();
}

template <typename TR, bool HF, bool XN, int HQ, bool XW = false>
int launch_any(const ConvGeom &g, int ksteps, const void *x, const void *wp, const void *bias, void *y, hipStream_t st) {
    if (g.KH <= 1 && ksteps <= 2) return launch_inst<TR, 1, 2, HF, XN, HQ, XW>(g, ksteps, x, wp, bias, y, st);
    if (g.KH <= 3 && ksteps <= 1) return launch_inst<TR, 3, 1, HF, XN, HQ, XW>(g, ksteps, x, wp, bias, y, st);
    return (int)hipErrorInvalidValue;
}

template <typename TR>
int launch_layout(const ConvGeom &g, int ksteps, bool height_fold, bool x_nchw, const void *x, const void *wp, const void *bias,
                  void *y, hipStream_t st) {
    if (height_fold) {
        // quads of four tiles where the two halves of the fold are whole waves, a thread of the write-out has its
        // two slots and the image is wide enough for 256-byte runs to exist
        // the columns in four parts and blocks of eight tiles (whole rows of images up to 256 columns wide) where a
        // part is whole waves, a thread of the write-out has its two slots and the image is wide enough to gain;
        // else in two parts and blocks of four tiles; else pairs
        const bool p4 = g.NCo % 256 == 0 && g.F % 8 == 0 && g.Hout > 128;
        const bool p2 = g.NCo % 128 == 0 && g.F % 4 == 0 && g.Hout > 64;
        if (p4) return x_nchw ? launch_any<TR, true, true, 4>(g, ksteps, x, wp, bias, y, st)
                              : launch_any<TR, true, false, 4>(g, ksteps, x, wp, bias, y, st);
        if (p2) return x_nchw ? launch_any<TR, true, true, 2>(g, ksteps, x, wp, bias, y, st)
                              : launch_any<TR, true, false, 2>(g, ksteps, x, wp, bias, y, st);
        return x_nchw ? launch_any<TR, true, true, 0>(g, ksteps, x, wp, bias, y, st)
                      : launch_any<TR, true, false, 0>(g, ksteps, x, wp, bias, y, st);
    }
    if (x_nchw) return launch_any<TR, false, false, 0, true>(g, ksteps, x, wp, bias, y, st);  // staged through LDS
    return launch_any<TR, false, false, 0>(g, ksteps, x, wp, bias, y, st);
}

}  // namespace

int fc_launch_conv_stream_nchw(foldconv_dtype_t dt, const ConvGeom &g, bool height_fold, bool x_nchw, const void *x,
                               const void *w_pack, const void *bias, void *y, void *stream) {
    int ksteps = 0;
    if (!fc_stream_nchw_ok(g, g.band, height_fold, &ksteps)) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    if (dt == FOLDCONV_F16) return launch_layout<F16Traits>(g, ksteps, height_fold, x_nchw, x, w_pack, bias, y, st);
    if (dt == FOLDCONV_BF16) return launch_layout<BF16Traits>(g, ksteps, height_fold, x_nchw, x, w_pack, bias, y, st);
    return (int)hipErrorInvalidValue;
}
