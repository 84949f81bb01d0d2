// Geometry of one (possibly folded) convolution as the kernels see it, plus
// the plan object behind the C ABI.  Host and device share this header.
//
// The folded problem is an implicit GEMM  y'^T[n][m] = sum_k w'[k][n] * A[m][k]
// with m = (image, output row, folded output column), n = g*C_out + co and
// k = (kh, e), where e is the "extended channel" coordinate of a tap relative
// to the folded pixel: e = d*F*C_in + c'.  Because x' is contiguous NHWC, the
// element for (m, kh, e) sits at   row(image, h+kh-pad_h) + w'*F*C_in + e,
// i.e. one contiguous window of the input row per (m, kh), and the matching
// filter row is  kh*KW'*F*C_in + (e - e_min).  Output slot g only has
// non-zero filter rows for e in [(g-p)*C_in, (g+KW-p)*C_in): the block band
// of the expanded filter (paper: Eq. "filter_construct" generalised to taps
// along the folded axis).
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "../../include/foldconv.h"

#if defined(__HIPCC__)
#define FC_HD __host__ __device__ inline
#else
#define FC_HD inline
#endif

struct ConvGeom {
    int N, H, Hout;
    int Wf;      // folded input width in pixels
    int Wf_out;  // folded output width in pixels
    int FC;      // channels per folded input pixel (F*C_in)
    int NCo;     // GEMM N: channels per folded output pixel (F*C_out)
    int Co;      // bias period (C_out)
    int C;       // original input channels (band arithmetic)
    int F, KH, KW, pad_h, pad_w;
    int epc;     // elements per operand chunk (what a lane loads of x' and of the filter per K-step half):
                 // 8 for the 16-bit types (16 bytes), 4 for fp32 (16 bytes); 8-byte chunks on the streaming kernel:
                 // 4 for a 16-bit layer whose F*C_in is a multiple of 4 but not of 8, 2 for an fp32 layer
                 // that walks fewer structural zeros that way (or whose F*C_in is a multiple of 2 only)
    int eb;      // bytes per element; stored output chunks are always 16 bytes = 16/eb elements
    int e_min, e_max;  // dense window of extended channels, [e_min, e_max)
    int kwin;          // e_max - e_min = KW'*FC = filter rows per kh
    int in_row;        // elements per input row  (Wf*FC)
    int out_row;       // elements per stored output row (W_out*Co, or Wf_out*NCo when kept folded)
    int relu, band, has_bias;
    int unpaced;       // leave the store stream of the streaming kernels unpaced (FOLDCONV_FLAG_UNPACED)
    int compact;       // the filter operand is the compact per-phase storage (see fc_compact_chunk)
    int cJ, cgcd;      // compact storage: chunks per (phase, kh), and gcd(C_in, 8)
    long long M;       // N*Hout*Wf_out
};

FC_HD int fc_floor_to(int x, int a) { int r = x % a; if (r < 0) r += a; return x - r; }
FC_HD int fc_ceil_to(int x, int a) { return fc_floor_to(x + a - 1, a); }

// Window [e_lo, e_hi) of extended channels that can hold a non-zero filter
// entry for output columns [n_lo, n_hi), rounded outwards to `align`.
FC_HD void fc_band_window(const ConvGeom &g, int n_lo, int n_hi, int align, int *e_lo, int *e_hi) {
    int lo = g.e_min, hi = g.e_max;
    if (g.band) {
        if (n_hi > g.NCo) n_hi = g.NCo;
        int g0 = n_lo / g.Co, g1 = (n_hi - 1) / g.Co;
        int blo = fc_floor_to((g0 - g.pad_w) * g.C, align);
        int bhi = fc_ceil_to((g1 + g.KW - g.pad_w) * g.C, align);
        if (blo > lo) lo = blo;
        if (bhi < hi) hi = bhi;
        if (hi < lo) hi = lo;
    }
    *e_lo = lo;
    *e_hi = hi;
}

// Compact storage of the expanded filter for the vector kernels.  Every output slot g
// uses the same KW*C_in x C_out matrix per kh (the non-zero blocks of w' are copies of the original
// taps; paper: "Potential Optimizations for Sparsity": keep only the non-zero blocks); slots differ
// only in where that matrix starts, a = (g-p)*C_in - e_min rows into the window.  In operand
// chunks of E = epc rows (ConvGeom.epc) the start falls on phase a mod E, a multiple of
// gcd(C_in, E), so one zero-padded copy per phase serves every slot:
//   cpk[ph][kh][j][co][i] = w[kh][t / C_in][t % C_in][co],  t = E*j + i - ph*gcd,  0 <= t < KW*C_in, else 0.
// Returns the chunk of cpk that equals rows [e_min+E*q, e_min+E*q+E) of column n of w', or -1 when
// those rows are structural zeros.
// E is a template argument (it must equal g.epc) so that the kernels divide by shifting.
template <int E>
FC_HD long long fc_compact_chunk(const ConvGeom &g, int kh, int q, int n) {
    static_assert(E == 2 || E == 4 || E == 8, "chunks of 2, 4 or 8 elements");
    constexpr int SH = E == 8 ? 3 : E == 4 ? 2 : 1;
    const int slot = n / g.Co, co = n - slot * g.Co;
    const int a = (slot - g.pad_w) * g.C - g.e_min;  // >= 0 because e_min <= -p*C_in
    const int j = q - (a >> SH);
    if (j < 0 || j >= g.cJ) return -1;
    return ((long long)(((a & (E - 1)) / g.cgcd) * g.KH + kh) * g.cJ + j) * g.Co + co;
}
// gcd(c, epc) for epc = 2, 4 or 8
FC_HD int fc_gcd_chunk(int c, int epc) {
    int d = epc;
    while (c % d != 0) d /= 2;
    return d;
}
FC_HD int fc_compact_phases(const ConvGeom &g) { return g.epc / g.cgcd; }

// How the persistent streaming kernels deal their 32-pixel M tiles to the XCDs (8 on MI355X; workgroup
// b runs on XCD b % parts, each XCD has its own L2).  Tiles go out in chunks of CH consecutive tiles, chunk c
// to XCD c % parts: neighbouring tiles share their input rows inside one L2, and at any moment the
// XCDs together write one compact region of y that moves through memory once (one contiguous range
// of tiles per XCD instead means eight write fronts far apart, which the memory system serves
// about 10 % slower).  An XCD holds J tiles at a time, as J/CH chunks that are `parts` chunks
// apart; slot j0 < J of XCD `part` starts at fc_deal_first_tile and then strides by parts*J tiles,
// so every tile below MT is visited exactly once.
struct FcDeal {
    unsigned parts;   // 1 (too few tiles to split), or the number of XCDs
    unsigned CH;      // tiles per chunk, divides J
    unsigned J;       // tiles in flight per XCD
    unsigned stride;  // parts * J
};
// slots: how many tiles one XCD's resident waves (or workgroups) can hold at a time.
FC_HD FcDeal fc_make_deal(unsigned MT, unsigned parts, unsigned slots, int KH, int Wf_out) {
    FcDeal d;
    d.parts = parts;
    const unsigned tpp = (MT + parts - 1) / parts;
    unsigned J = slots < 1 ? 1 : slots;
    if (J > tpp) J = tpp;
    if (J < 1) J = 1;
    unsigned CH = 1;
    if (parts > 1) {
        // a chunk spans four output rows or more: the rows it shares with its neighbours (fetched
        // into two L2s) stay a small part of what it reads
        CH = 2;
        while (KH > 1 && CH < 1024 && 32ll * CH < 4ll * Wf_out) CH *= 2;
        while (CH > J || (CH > 1 && MT < 4 * parts * CH)) CH /= 2;
        J -= J % CH;
    }
    d.CH = CH;
    d.J = J;
    d.stride = J * parts;
    return d;
}
FC_HD unsigned fc_deal_first_tile(const FcDeal &d, unsigned part, unsigned j0) {
    const unsigned jc = j0 / d.CH;
    return (d.parts * jc + part) * d.CH + (j0 - jc * d.CH);
}

enum { FC_KERNEL_GATHER = 0, FC_KERNEL_TILED = 1, FC_KERNEL_STREAM = 2 };

struct FcStamps {
    const void *ws[4];
    unsigned next;
};
inline bool fc_stamped(const FcStamps *s, const void *ws) {
    if (!ws) return false;
    for (int i = 0; i < 4; ++i)
        if (__atomic_load_n(&s->ws[i], __ATOMIC_RELAXED) == ws) return true;
    return false;
}
inline void fc_stamp(FcStamps *s, const void *ws) {
    if (fc_stamped(s, ws)) return;
    const unsigned i = __atomic_fetch_add(&s->next, 1u, __ATOMIC_RELAXED) & 3u;
    __atomic_store_n(&s->ws[i], ws, __ATOMIC_RELAXED);
}

struct foldconv_plan_s {
    uint32_t magic;
    foldconv_shapes_t s;
    ConvGeom fold;  // the folded problem (band/relu/out_row/has_bias filled per call)
    ConvGeom padc;  // the zero-padded problem, F = 1, C = C_pad
    // byte offsets inside the padded-path workspace
    size_t ws_xpad, ws_wpad, ws_wpack, ws_bpad, ws_ypad;
    int fold_axis;  // FOLDCONV_FOLD_W, or FOLDCONV_FOLD_H for a channels-first plan built on the transposed image
    // Where this plan wrote a kernel-order filter (foldconv_pack_filter, foldconv_forward without
    // FOLDCONV_FLAG_FILTER_PACKED, foldconv_pack_filter_compact, conv_padded_forward): a later call that
    // claims a prepared filter in a workspace the plan never wrote is refused instead of computing on
    // garbage.  The last four workspaces of each kind are remembered (one plan may serve several streams,
    // each with its own copy); relaxed atomics, plans may be shared between threads.
    FcStamps packed_ws, compact_ws, padded_ws;
};

#define FOLDCONV_MAGIC 0xF01DC0DEu
