// LDS-tiled MFMA convolution for layers whose K extent is too large for the
// filter-stationary streaming kernel (tens to hundreds of 16-wide K-steps):
// there the matrix cores, not HBM, bound the layer.
//
// One 256-thread workgroup (4 waves, 2 x 2) computes a BN (output columns n)
// x 128 (folded output pixels m) tile of y'^T, BN = 128 or 256; each wave a
// (BN/2) x 64 quadrant as TN x 2 MFMA tiles of 32 x 32 (TN = 2 or 4: the wider
// tile halves the LDS reads and the input re-reads per MFMA and is used when
// there are enough output columns to fill it).  K = (kh, extended channel e) is walked in
// blocks of 32 elements (two MFMA K-steps), restricted to the band of w' that
// can be non-zero for the tile's output slots (paper: Eq. "filter_construct";
// off-band blocks are structural zeros) unless the dense walk is asked for.
// Both operands are staged through LDS in MFMA operand order, one 16-byte
// chunk (8 consecutive K values of one row/column) per lane access:
//   filter: pack[kh][q][n][8] rows copied as they are (coalesced),
//   input:  the window chunk [e, e+8) of each pixel's input row, a 16-byte
//           range-checked buffer load (zero padding = out-of-range offset).
// Global loads for block i+1 are issued before the MFMAs of block i and
// written to the other LDS stage afterwards: one barrier per K block.
// Epilogue: bias as a rank-1 MFMA, ReLU, one rounding, transpose through LDS,
// 16-byte row-contiguous stores with the reconstruct step fused in.
// paper: Eq. "new_conv_H", Eq. "bias_construct", Reconstruct step.
#include <hip/hip_runtime.h>

#include "launch.h"
#include "mfma_types.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int BM = 128, BK = 32;
constexpr int QPB = BK / 8;                 // 16-byte chunks per row per K block
constexpr unsigned kOutOfRange = 0x80000000u;

// LDS geometry for a tile of BN output columns
template <int BN>
struct TileLds {
    // bytes of one chunk plane; the pad staggers the planes so that the 16 lanes of a staging write
    // (QPB chunks x 16/QPB pixels) fall on 16 distinct bank groups
    static constexpr int PLANE_F = BN * 16 + 256 / QPB;
    static constexpr int PLANE_I = BM * 16 + 256 / QPB;
    static constexpr int STAGE = QPB * (PLANE_F + PLANE_I);  // filter planes then input planes
    static constexpr int EPITCH = BN * 2 + 16;               // bytes per row of the transposed output half-tile
    static constexpr int EBYTES = 64 * EPITCH;               // the epilogue handles 64 pixels at a time
    static constexpr int BYTES = (2 * STAGE > EBYTES) ? 2 * STAGE : EBYTES;
};

template <typename TR>
__device__ __forceinline__ unsigned pack2t(float a, float b);
template <>
__device__ __forceinline__ unsigned pack2t<F16Traits>(float a, float b) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 v = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(unsigned, v);
}
template <>
__device__ __forceinline__ unsigned pack2t<BF16Traits>(float a, float b) {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    b2 v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(unsigned, v);
}

struct TiledArgs {
    unsigned tiles_n, tiles_m;
    unsigned total;      // tiles_n * tiles_m
    unsigned per_xcd;    // ceil(total / 8)
    unsigned x_bytes, wp_bytes;
};

template <typename TR, int TN, bool RELU>
__global__ void __launch_bounds__(256, 2)
conv_tiled_kernel(ConvGeom g, TiledArgs a, const typename TR::T *__restrict__ x, const u32x4 *__restrict__ wp,
                  const typename TR::T *__restrict__ bias, typename TR::T *__restrict__ y) {
    using T = typename TR::T;
    using Vec = typename TR::Vec;
    constexpr int BN = 64 * TN;
    using L = TileLds<BN>;
    constexpr int PLANE_F = L::PLANE_F, PLANE_I = L::PLANE_I, STAGE = L::STAGE, EPITCH = L::EPITCH;
    __shared__ __attribute__((aligned(16))) unsigned char lds[L::BYTES];

    // Workgroup b runs on XCD b % 8.  Each XCD takes one contiguous range of tiles, N tiles
    // fastest, so the tiles that share an input window meet in one L2.
    const unsigned tile = (blockIdx.x % 8u) * a.per_xcd + blockIdx.x / 8u;
    if (blockIdx.x / 8u >= a.per_xcd || tile >= a.total) return;  // uniform per workgroup
    const unsigned tm = tile / a.tiles_n, tn = tile - tm * a.tiles_n;
    const int n0 = (int)tn * BN;
    const unsigned m0 = tm * BM;

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int r = lane & 31, hf = lane >> 5;
    const int wn = wave & 1, wm = wave >> 1;

    int e_lo, e_hi;
    fc_band_window(g, n0, n0 + BN, 8, &e_lo, &e_hi);
    const int kblocks = (e_hi - e_lo + BK - 1) / BK;  // per kh
    const int T_total = g.KH * kblocks;
    const int q_per_kh = g.kwin / 8;

    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<T *>(x), 0, (int)a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(const_cast<u32x4 *>(wp), 0, (int)a.wp_bytes, 0x00020000);

    // ---- this thread's share of the staging loads -----------------------------
    // input: chunk column qi of NI pixels, one 16-byte chunk each
    constexpr int NI = (BM * QPB) / 256;   // input chunks per thread per K block
    constexpr int NF = (BN * QPB) / 256;   // filter chunks per thread per K block
    constexpr int MSTEP = 256 / QPB;       // pixels covered by one pass of the 256 threads
    const int qi = t & (QPB - 1);
    int pix[NI], ho_[NI], col_[NI];
    bool vm[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const unsigned m = m0 + (unsigned)(t / QPB) + (unsigned)(MSTEP * i);
        vm[i] = m < (unsigned)g.M;
        const unsigned mm = vm[i] ? m : 0u;
        const unsigned wo = mm % (unsigned)g.Wf_out;
        const unsigned rowid = mm / (unsigned)g.Wf_out;
        const unsigned ho = rowid % (unsigned)g.Hout;
        const unsigned img = rowid / (unsigned)g.Hout;
        ho_[i] = (int)ho;
        col_[i] = (int)wo * g.FC + 8 * qi;
        pix[i] = ((int)(img * (unsigned)g.H + ho) - g.pad_h) * g.in_row + col_[i];
    }
    // filter: BN columns x QPB planes = NF chunks per thread, column-contiguous across threads
    // The chunk for window chunk q of a column sits at  fbase + (kh*f_jmax + (q - fj0)) * f_stride
    // when 0 <= q - fj0 < f_jmax.  Packed w': one run of q_per_kh chunks per kh, column stride NCo.
    // Compact storage: the column's slot fixes the phase copy and the first window chunk its tap
    // matrix reaches (fc_compact_chunk); chunks outside are structural zeros.
    int nf[NF], qf[NF], fbase[NF], fj0[NF];
    bool vn[NF];
    const int f_jmax = g.compact ? g.cJ : q_per_kh;
    const int f_stride = g.compact ? g.Co : g.NCo;
#pragma unroll
    for (int i = 0; i < NF; ++i) {
        const int idx = t + 256 * i;
        nf[i] = idx % BN;
        qf[i] = idx / BN;
        vn[i] = n0 + nf[i] < g.NCo;
        const int n = vn[i] ? n0 + nf[i] : 0;
        if (g.compact) {
            const int slot = n / g.Co, co = n - slot * g.Co;
            const int a = (slot - g.pad_w) * g.C - g.e_min;
            fj0[i] = a >> 3;
            fbase[i] = ((a & 7) / g.cgcd) * g.KH * g.cJ * g.Co + co;
        } else {
            fj0[i] = 0;
            fbase[i] = n;
        }
    }

    // Two register sets: the loads of block i+2 are issued while block i is computed and are
    // written to LDS one step later, so they have a whole step of MFMAs (of this and of the
    // co-resident workgroup) to land.
    struct StageRegs {
        u32x4 ri[NI], rf[NF];
    };
    StageRegs ra, rb;
    int kh_l = 0, kb_l = 0;  // next block to load
    auto load_block = [&](StageRegs &rg) {
        const bool live = kh_l < g.KH;
        const int kh = live ? kh_l : 0;
        const int e0 = live ? e_lo + kb_l * BK : e_hi;  // past the window: every lane out of range
        u32x4 (&ri)[NI] = rg.ri;
        u32x4 (&rf)[NF] = rg.rf;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int hi = ho_[i] + kh - g.pad_h;
            const int e = e0 + 8 * qi;
            const int col = col_[i] + e0;
            const bool ok = vm[i] && hi >= 0 && hi < g.H && e < e_hi && col >= 0 && col < g.in_row;
            const unsigned off = ok ? 2u * (unsigned)(pix[i] + kh * g.in_row + e0) : kOutOfRange;
            ri[i] = __builtin_amdgcn_raw_buffer_load_b128(xr, off, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < NF; ++i) {
            const int e = e0 + 8 * qf[i];
            const int j = ((e - g.e_min) >> 3) - fj0[i];
            const bool ok = vn[i] && e < e_hi && j >= 0 && j < f_jmax;
            const unsigned off = ok ? 16u * ((unsigned)fbase[i] + (unsigned)(kh * f_jmax + j) * (unsigned)f_stride) : kOutOfRange;
            rf[i] = __builtin_amdgcn_raw_buffer_load_b128(wr, off, 0, 0);
        }
        if (++kb_l == kblocks) {
            kb_l = 0;
            ++kh_l;
        }
    };
    auto store_block = [&](const StageRegs &rg, int stage) {
        const u32x4 (&ri)[NI] = rg.ri;
        const u32x4 (&rf)[NF] = rg.rf;
        unsigned char *sf = lds + stage * STAGE;
        unsigned char *si = sf + QPB * PLANE_F;
#pragma unroll
        for (int i = 0; i < NI; ++i)
            *reinterpret_cast<u32x4 *>(si + qi * PLANE_I + (t / QPB + MSTEP * i) * 16) = ri[i];
#pragma unroll
        for (int i = 0; i < NF; ++i)
            *reinterpret_cast<u32x4 *>(sf + qf[i] * PLANE_F + nf[i] * 16) = rf[i];
    };

    // ---- accumulators, initialised with the bias through a rank-1 MFMA ----------
    floatx16_t acc[TN][2];
    {
        Vec ones;
#pragma unroll
        for (int i = 0; i < 8; ++i) ones[i] = (T)0.0f;
        if (hf == 0) ones[0] = (T)1.0f;
        floatx16_t zero;
#pragma unroll
        for (int i = 0; i < 16; ++i) zero[i] = 0.0f;
#pragma unroll
        for (int nt = 0; nt < TN; ++nt) {
            Vec bf;
#pragma unroll
            for (int i = 0; i < 8; ++i) bf[i] = (T)0.0f;
            const int n = n0 + wn * (BN / 2) + nt * 32 + r;
            if (g.has_bias && hf == 0 && n < g.NCo) bf[0] = bias[n % g.Co];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) acc[nt][mt] = TR::mfma(bf, ones, zero);
        }
    }

    // ---- K loop -----------------------------------------------------------------
    auto compute = [&](int stage) {
        const unsigned char *sf = lds + stage * STAGE;
        const unsigned char *si = sf + QPB * PLANE_F;
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            const int qc = 2 * s + hf;
            Vec af[TN], bfv[2];
#pragma unroll
            for (int nt = 0; nt < TN; ++nt)
                af[nt] = *reinterpret_cast<const Vec *>(sf + qc * PLANE_F + (wn * (BN / 2) + nt * 32 + r) * 16);
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
                bfv[mt] = *reinterpret_cast<const Vec *>(si + qc * PLANE_I + (wm * 64 + mt * 32 + r) * 16);
#pragma unroll
            for (int nt = 0; nt < TN; ++nt)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) acc[nt][mt] = TR::mfma(af[nt], bfv[mt], acc[nt][mt]);
        }
    };
    // Blocks past the end load nothing (out-of-range offsets) and are never computed.
    load_block(ra);
    load_block(rb);
    store_block(ra, 0);
    __syncthreads();
    for (int it = 0; it < T_total; it += 2) {
        load_block(ra);        // block it+2
        compute(0);            // block it
        store_block(rb, 1);    // block it+1
        __syncthreads();
        if (it + 1 >= T_total) break;
        load_block(rb);        // block it+3
        compute(1);            // block it+1
        store_block(ra, 0);    // block it+2
        __syncthreads();
    }

    // ---- epilogue: round, ReLU, transpose through LDS (stages are free after the last barrier),
    // 64 pixels (one MFMA tile row per wave) at a time ----
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        if (mt) __syncthreads();  // the first half has been read out
#pragma unroll
        for (int nt = 0; nt < TN; ++nt)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                u32x2 pk = {pack2t<TR>(acc[nt][mt][4 * q], acc[nt][mt][4 * q + 1]),
                            pack2t<TR>(acc[nt][mt][4 * q + 2], acc[nt][mt][4 * q + 3])};
                if (RELU) {
                    typedef short s16x4 __attribute__((ext_vector_type(4)));
                    const s16x4 z = {0, 0, 0, 0};
                    pk = __builtin_bit_cast(u32x2, __builtin_elementwise_max(__builtin_bit_cast(s16x4, pk), z));
                }
                const int row = wm * 32 + r;  // pixel wm*64 + mt*32 + r of the tile
                const int col = wn * (BN / 2) + nt * 32 + 8 * q + 4 * hf;
                *reinterpret_cast<u32x2 *>(lds + row * EPITCH + col * 2) = pk;
            }
        __syncthreads();
        constexpr int CPR = BN / 8;  // 16-byte chunks per row
#pragma unroll
        for (int i = 0; i < (64 * CPR) / 256; ++i) {
            const int idx = i * 256 + t;
            const int row = idx / CPR, ch = idx % CPR;
            const unsigned m = m0 + (unsigned)((row >> 5) * 64 + mt * 32 + (row & 31));
            const int n = n0 + 8 * ch;
            if (m < (unsigned)g.M && n < g.NCo) {
                const unsigned wo = m % (unsigned)g.Wf_out;
                const unsigned rowid = m / (unsigned)g.Wf_out;
                const unsigned oc = wo * (unsigned)g.NCo + (unsigned)n;
                if (oc + 8u <= (unsigned)g.out_row) {
                    const u32x4 v = *reinterpret_cast<const u32x4 *>(lds + row * EPITCH + ch * 16);
                    const unsigned long long off8 = ((unsigned long long)rowid * (unsigned)g.out_row + oc) >> 3;
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(y) + off8);
                }
            }
        }
    }
}

template <typename TR, int TN>
int launch(const ConvGeom &g, const void *x, const void *wp, const void *bias, void *y, hipStream_t st) {
    using T = typename TR::T;
    constexpr int BN = 64 * TN;
    TiledArgs a;
    a.tiles_n = (unsigned)((g.NCo + BN - 1) / BN);
    a.tiles_m = (unsigned)((g.M + BM - 1) / BM);
    const unsigned long long total = (unsigned long long)a.tiles_n * a.tiles_m;
    if (total > 0x7fffff00ull) return (int)hipErrorInvalidValue;
    a.total = (unsigned)total;
    a.per_xcd = (a.total + 7) / 8;
    a.x_bytes = (unsigned)((long long)g.N * g.H * g.in_row * (long long)sizeof(T));
    a.wp_bytes = g.compact ? (unsigned)((long long)fc_compact_phases(g) * g.KH * g.cJ * g.Co * 16)
                           : (unsigned)((long long)g.KH * g.kwin * g.NCo * (long long)sizeof(T));
    const unsigned blocks = a.per_xcd * 8;
    if (g.relu)
        conv_tiled_kernel<TR, TN, true><<<blocks, 256, 0, st>>>(g, a, (const T *)x, (const u32x4 *)wp, (const T *)bias, (T *)y);
    else
        conv_tiled_kernel<TR, TN, false><<<blocks, 256, 0, st>>>(g, a, (const T *)x, (const u32x4 *)wp, (const T *)bias, (T *)y);
    return (int)hipGetLastError();
}

template <typename TR>
int launch_any(const ConvGeom &g, const void *x, const void *wp, const void *bias, void *y, hipStream_t st) {
    return fc_tiled_bn(g) == 256 ? launch<TR, 4>(g, x, wp, bias, y, st) : launch<TR, 2>(g, x, wp, bias, y, st);
}

}  // namespace

int fc_launch_conv_tiled(foldconv_dtype_t dt, const ConvGeom &g, const void *x, const void *w_pack, const void *bias,
                         void *y, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    if (dt == FOLDCONV_F16) return launch_any<F16Traits>(g, x, w_pack, bias, y, st);
    if (dt == FOLDCONV_BF16) return launch_any<BF16Traits>(g, x, w_pack, bias, y, st);
    return (int)hipErrorInvalidValue;
}
