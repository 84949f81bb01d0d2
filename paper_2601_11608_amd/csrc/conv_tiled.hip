// LDS-tiled MFMA convolution for layers whose K extent is too large for the
// filter-stationary streaming kernel (tens to hundreds of 16-wide K-steps):
// there the matrix cores, not HBM, bound the layer.
//
// One workgroup of 2 x WM waves computes a BN (output columns n) x BM (folded
// output pixels m) tile of y'^T, BN = 128 or 256, BM = 64*WM (128 as built);
// each wave a (BN/2) x 64 part as TN x 2 MFMA tiles of 32 x 32 (TN = 2 or 4: the
// wider tile halves the LDS reads and the input re-reads per MFMA and is used when
// there are enough output columns to fill it).  K = (kh, extended channel e) is walked in
// blocks of 32 elements (two MFMA K-steps), restricted to the band of w' that
// can be non-zero for the tile's output slots (paper: Eq. "filter_construct";
// off-band blocks are structural zeros) unless the dense walk is asked for.
// Both operands are staged through LDS in MFMA operand order, one 16-byte
// chunk (8 consecutive K values of one row/column) per lane access:
//   filter: pack[kh][q][n][8] rows copied as they are (coalesced),
//   input:  the window chunk [e, e+8) of each pixel's input row, a 16-byte
//           range-checked buffer load (zero padding = out-of-range offset).
// The K loop is one software pipeline: while block b is multiplied, the global
// loads of block b+2 and the LDS writes of block b+1 are issued one per MFMA
// step, and the LDS fragment reads run two steps ahead of the MFMAs that use
// them; one barrier per K block.  The staging loads are inline assembly with
// explicit wait counts (checked by a test that walks the generated code).
// Epilogue: bias as a rank-1 MFMA, ReLU, one rounding, transpose through LDS,
// 16-byte row-contiguous stores with the reconstruct step fused in.
// paper: Eq. "new_conv_H", Eq. "bias_construct", Reconstruct step.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "launch.h"
#include "mfma_types.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int BK = 32;
constexpr int QPB = BK / 8;                 // 16-byte chunks per row per K block
constexpr unsigned kOutOfRange = 0x80000000u;

// LDS geometry for a tile of BN output columns x BM pixels
template <int BN, int BM>
struct TileLds {
    // bytes of one chunk plane; the pad staggers the planes so that the 16 lanes of a staging write
    // (QPB chunks x 16/QPB pixels) fall on 16 distinct bank groups
    static constexpr int PLANE_F = BN * 16 + 256 / QPB;
    static constexpr int PLANE_I = BM * 16 + 256 / QPB;
    static constexpr int STAGE = QPB * (PLANE_F + PLANE_I);  // filter planes then input planes
    static constexpr int EPITCH = BN * 2 + 16;               // bytes per row of the transposed output half-tile
    static constexpr int EBYTES = (BM / 2) * EPITCH;         // the epilogue handles one 32-pixel MFMA row per wave at a time
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

template <typename TR, int TN, int WM, bool RELU>
__global__ void __launch_bounds__(128 * WM, WM == 2 ? 2 : 1)
conv_tiled_kernel(ConvGeom g, TiledArgs a, const typename TR::T *__restrict__ x, const u32x4 *__restrict__ wp,
                  const typename TR::T *__restrict__ bias, typename TR::T *__restrict__ y) {
    using T = typename TR::T;
    using Vec = typename TR::Vec;
    constexpr int BN = 64 * TN;        // two wave columns of TN MFMA tiles
    constexpr int BM = 64 * WM;        // WM wave rows of two MFMA tiles
    constexpr int THREADS = 128 * WM;  // 2 x WM waves
    using L = TileLds<BN, BM>;
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

    // Range-checked raw buffer resources (byte offsets; an offset beyond the extent reads as zero).
    // They are built by hand as SGPR quads because the staging loads below are inline assembly.
    auto make_srd = [](const void *p, unsigned bytes) {
        const unsigned long long a = (unsigned long long)p;
        u32x4 r;
        r[0] = __builtin_amdgcn_readfirstlane((unsigned)a);
        r[1] = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32) & 0xffffu);
        r[2] = __builtin_amdgcn_readfirstlane(bytes);
        r[3] = __builtin_amdgcn_readfirstlane(0x00020000u);
        return r;
    };
    u32x4 xr = make_srd(x, a.x_bytes);  // not const: the generic lambdas below must capture them for asm operands
    u32x4 wr = make_srd(wp, a.wp_bytes);

    // ---- this thread's share of the staging loads -----------------------------
    // input: chunk column qi of NI pixels, one 16-byte chunk each
    constexpr int NI = (BM * QPB) / THREADS;   // input chunks per thread per K block
    constexpr int NF = (BN * QPB) / THREADS;   // filter chunks per thread per K block
    constexpr int NL = NI + NF;                // staging loads per thread per K block
    constexpr int MSTEP = THREADS / QPB;       // pixels covered by one pass of the workgroup
    const int qi = t & (QPB - 1);
    int pix[NI], ho_[NI], col_[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const unsigned m = m0 + (unsigned)(t / QPB) + (unsigned)(MSTEP * i);
        const bool vm = m < (unsigned)g.M;
        const unsigned mm = vm ? m : 0u;
        const unsigned wo = mm % (unsigned)g.Wf_out;
        const unsigned rowid = mm / (unsigned)g.Wf_out;
        const unsigned ho = rowid % (unsigned)g.Hout;
        const unsigned img = rowid / (unsigned)g.Hout;
        ho_[i] = vm ? (int)ho : -0x40000000;  // a pixel past the end fails every row test below
        col_[i] = (int)wo * g.FC + 8 * qi;
        pix[i] = ((int)(img * (unsigned)g.H + ho) - g.pad_h) * g.in_row + col_[i];
    }
    // The chunk for window chunk q of a column sits at  fbase + (kh*f_jmax + (q - fj0)) * f_stride
    // when 0 <= q - fj0 < f_jmax.  Packed w': one run of q_per_kh chunks per kh, column stride NCo.
    // Compact storage: the column's slot fixes the phase copy and the first window chunk its tap
    // matrix reaches (fc_compact_chunk); chunks outside are structural zeros.
    int nf[NF], qf[NF], fbase[NF], fj0[NF];
    const int f_jmax = g.compact ? g.cJ : q_per_kh;
    const int f_stride = g.compact ? g.Co : g.NCo;
#pragma unroll
    for (int i = 0; i < NF; ++i) {
        const int idx = t + THREADS * i;
        nf[i] = idx % BN;
        qf[i] = idx / BN;
        const bool vn = n0 + nf[i] < g.NCo;
        const int n = vn ? n0 + nf[i] : 0;
        if (g.compact) {
            const int slot = n / g.Co, co = n - slot * g.Co;
            const int a_g = (slot - g.pad_w) * g.C - g.e_min;
            fj0[i] = a_g >> 3;
            fbase[i] = ((a_g & 7) / g.cgcd) * g.KH * g.cJ * g.Co + co;
        } else {
            fj0[i] = 0;
            fbase[i] = n;
        }
        if (!vn) fj0[i] = 0x40000000;  // a column past the end fails the chunk range test below
    }

    // Staging loads are issued from inline assembly and waited for with explicit counts: left to
    // itself the compiler wraps every address select in a branch and waits for the loads of the
    // previous K block at the top of the loop.  Vector-memory loads return in issue order, so
    // "at most NL outstanding" means every load older than the NL newest has landed.
    // Nothing else in the K loop touches vector memory.  The pipeline below has one code path:
    // blocks past the end are issued with every lane out of range (no memory traffic, zeros
    // returned) and committed to a stage nobody reads; what is still in flight when the loop
    // ends is drained before any register is reused.
    struct StageRegs {
        u32x4 r[NL];
    };
    StageRegs ra, rb;
    int kh_l = 0, kb_l = 0;  // next block to issue
    int is_kh = 0, is_e0 = 0;  // block being issued (wave-uniform)
    auto issue_begin = [&]() {
        const bool live = kh_l < g.KH;
        is_kh = live ? kh_l : 0;
        is_e0 = live ? e_lo + kb_l * BK : e_hi;  // past the window: every lane out of range
        if (++kb_l == kblocks) {
            kb_l = 0;
            ++kh_l;
        }
    };
    // load number `idx` of the block (a constant once the caller's loop is unrolled): NI input
    // chunks, then NF filter chunks
    auto issue_one = [&](StageRegs &rg, int idx) {
        const int kh = is_kh, e0 = is_e0;
        if (idx < NI) {
            const int i = idx < NI ? idx : 0;
            const int hi = ho_[i] + kh - g.pad_h;
            const int col = col_[i] + e0;
            const int ok = (int)((unsigned)hi < (unsigned)g.H) & (int)((unsigned)col < (unsigned)g.in_row) &
                           (int)(e0 + 8 * qi < e_hi);
            const unsigned val = 2u * (unsigned)(pix[i] + kh * g.in_row + e0);
            const unsigned off = ok ? val : kOutOfRange;
            asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(rg.r[i]) : "v"(off), "s"(xr) : "memory");
        } else {
            const int i = idx < NI ? 0 : idx - NI;
            const int e = e0 + 8 * qf[i];
            const int j = ((e - g.e_min) >> 3) - fj0[i];
            const int ok = (int)(e < e_hi) & (int)((unsigned)j < (unsigned)f_jmax);
            const unsigned val = 16u * ((unsigned)fbase[i] + (unsigned)(kh * f_jmax + j) * (unsigned)f_stride);
            const unsigned off = ok ? val : kOutOfRange;
            asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(rg.r[NI + i]) : "v"(off), "s"(wr) : "memory");
        }
    };
    auto issue = [&](StageRegs &rg) {
        issue_begin();
#pragma unroll
        for (int k = 0; k < NL; ++k) issue_one(rg, k);
    };
    // One wait that names every register of the set, so the set stays allocated until it has landed:
    // returns once at most `count` younger loads are outstanding.
    auto wait_set = [&](StageRegs &rg, auto count) {
        constexpr int N = decltype(count)::value;
        if constexpr (NL == 4)
            asm volatile("s_waitcnt vmcnt(%4)" : "+v"(rg.r[0]), "+v"(rg.r[1]), "+v"(rg.r[2]), "+v"(rg.r[3]) : "n"(N) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(%6)"
                         : "+v"(rg.r[0]), "+v"(rg.r[1]), "+v"(rg.r[2]), "+v"(rg.r[3]), "+v"(rg.r[4]), "+v"(rg.r[5])
                         : "n"(N) : "memory");
    };
    static_assert(NL == 4 || NL == 6, "wait_set lists the staging registers explicitly");
    auto commit_one = [&](StageRegs &rg, int stage, int idx) {
        unsigned char *sf = lds + stage * STAGE;
        unsigned char *si = sf + QPB * PLANE_F;
        if (idx < NI) {
            const int i = idx < NI ? idx : 0;
            *reinterpret_cast<u32x4 *>(si + qi * PLANE_I + (t / QPB + MSTEP * i) * 16) = rg.r[i];
        } else {
            const int i = idx < NI ? 0 : idx - NI;
            *reinterpret_cast<u32x4 *>(sf + qf[i] * PLANE_F + nf[i] * 16) = rg.r[NI + i];
        }
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
    // One K block = BK/16 MFMA K-steps x TN filter fragments, walked as a rolling pipeline: the
    // fragment for step k+2 is requested from LDS before the two MFMAs of step k are issued, so
    // an LDS round trip has 128 cycles of matrix work to hide behind.  The staging traffic of the
    // blocks ahead is woven into the same instruction stream instead of following it: the global
    // loads of block b+2 go out after the first step, and the LDS writes of block b+1 (into the
    // stage nobody reads during this block) after the middle one, so they complete under the
    // remaining MFMAs and the wave reaches the barrier with nothing left to wait for.  The
    // scheduling fences keep the compiler from regrouping any of it.
    auto block = [&](int stage, StageRegs &next2, StageRegs &next1) {
        const unsigned char *sf = lds + stage * STAGE;
        const unsigned char *si = sf + QPB * PLANE_F;
        constexpr int KS = BK / 16, STEPS = KS * TN;
        constexpr int W = STEPS - NL;  // first step that writes to LDS (earlier placements measured the same)
        static_assert(W >= 0 && W + NL <= STEPS && NL <= STEPS, "one staging load and one staging write per step");
        Vec fr[3], in[KS][2];
        auto read_f = [&](int k) {
            const int qc = 2 * (k / TN) + hf;
            return *reinterpret_cast<const Vec *>(sf + qc * PLANE_F + (wn * (BN / 2) + (k % TN) * 32 + r) * 16);
        };
        auto read_i = [&](int ks, int mt) {
            const int qc = 2 * ks + hf;
            return *reinterpret_cast<const Vec *>(si + qc * PLANE_I + (wm * 64 + mt * 32 + r) * 16);
        };
        issue_begin();
        in[0][0] = read_i(0, 0);
        in[0][1] = read_i(0, 1);
        fr[0] = read_f(0);
        fr[1] = read_f(1);
#pragma unroll
        for (int k = 0; k < STEPS; ++k) {
            if (k + 2 < STEPS) fr[(k + 2) % 3] = read_f(k + 2);
#pragma unroll
            for (int ks = 1; ks < KS; ++ks)
                if (k == ks * TN - 2) {
                    in[ks][0] = read_i(ks, 0);
                    in[ks][1] = read_i(ks, 1);
                }
            __builtin_amdgcn_sched_barrier(0);
            const int ks = k / TN, nt = k % TN;
            acc[nt][0] = TR::mfma(fr[k % 3], in[ks][0], acc[nt][0]);
            acc[nt][1] = TR::mfma(fr[k % 3], in[ks][1], acc[nt][1]);
            __builtin_amdgcn_sched_barrier(0);
            // staging work of this step: one global load of block b+2, and from step W on one LDS
            // write of block b+1 (its loads are older than the k+1 loads of b+2 issued so far)
            if (k < NL) issue_one(next2, k);
            if (k == W) wait_set(next1, std::integral_constant<int, (W + 1 < NL ? W + 1 : NL)>{});
            if (k >= W && k < W + NL) commit_one(next1, stage ^ 1, k - W);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // Software pipeline over K blocks b = 0 .. T_total-1 (set and stage of block b: b & 1): while
    // block b is multiplied, block b+2 is requested from memory and block b+1 is written to LDS.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // nothing the compiler tracks may be in flight
    issue(ra);
    issue(rb);
    wait_set(ra, std::integral_constant<int, NL>{});
#pragma unroll
    for (int k = 0; k < NL; ++k) commit_one(ra, 0, k);
    __syncthreads();
    for (int it = 0; it < T_total; it += 2) {
        block(0, ra, rb);  // multiply block it, request it+2 into ra, write it+1 from rb to stage 1
        __syncthreads();
        if (it + 1 >= T_total) break;
        block(1, rb, ra);  // multiply block it+1, request it+3 into rb, write it+2 from ra to stage 0
        __syncthreads();
    }
    // the set issued last was never committed: let it land before its registers are reused
    wait_set(ra, std::integral_constant<int, 0>{});
    wait_set(rb, std::integral_constant<int, 0>{});

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
        for (int i = 0; i < (32 * WM * CPR) / THREADS; ++i) {
            const int idx = i * THREADS + t;
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

template <typename TR, int TN, int WM>
int launch(const ConvGeom &g, const void *x, const void *wp, const void *bias, void *y, hipStream_t st) {
    using T = typename TR::T;
    constexpr int BN = 64 * TN, BM = 64 * WM, THREADS = 128 * WM;
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
        conv_tiled_kernel<TR, TN, WM, true><<<blocks, THREADS, 0, st>>>(g, a, (const T *)x, (const u32x4 *)wp, (const T *)bias, (T *)y);
    else
        conv_tiled_kernel<TR, TN, WM, false><<<blocks, THREADS, 0, st>>>(g, a, (const T *)x, (const u32x4 *)wp, (const T *)bias, (T *)y);
    return (int)hipGetLastError();
}

template <typename TR>
int launch_any(const ConvGeom &g, const void *x, const void *wp, const void *bias, void *y, hipStream_t st) {
    // A 256 x 256 tile on eight waves (WM = 4) moves a third fewer operand bytes per multiply but
    // measured the same as 256 x 128 on the layers it fits, so only WM = 2 is instantiated.
    return fc_tiled_bn(g) == 256 ? launch<TR, 4, 2>(g, x, wp, bias, y, st) : launch<TR, 2, 2>(g, x, wp, bias, y, st);
}

}  // namespace

int fc_launch_conv_tiled(foldconv_dtype_t dt, const ConvGeom &g, const void *x, const void *w_pack, const void *bias,
                         void *y, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    if (dt == FOLDCONV_F16) return launch_any<F16Traits>(g, x, w_pack, bias, y, st);
    if (dt == FOLDCONV_BF16) return launch_any<BF16Traits>(g, x, w_pack, bias, y, st);
    return (int)hipErrorInvalidValue;
}
