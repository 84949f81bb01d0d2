// Filter-stationary streaming MFMA convolution with the input tile staged through LDS:
// the dense walk of the expanded filter (every K-step of w', structural zeros included)
// for layers whose whole K extent fits the register file.
//
// The plain streaming kernel lets every wave fetch its own input fragments through the
// vector L1.  That is right for the band walk (three fragments per tile), but on the dense
// walk a wave needs KH*KW'*F*C_in/16 fragments per tile (27 on the 224x224 C_in = 3 layer)
// for only two MFMAs each, and four waves per compute unit then ask the L1 for 64 bytes
// per clock, all it can deliver.  Here the four waves of a workgroup (256 output columns,
// 64 per wave, filter fragments for the full K extent resident in registers) share one
// 32-pixel input tile: it is brought into LDS once per workgroup by buffer loads that
// deposit straight into LDS, laid out so that one load instruction writes exactly one MFMA
// operand (64 lanes x 16 bytes) and every fragment read is a conflict-free 16-byte LDS read.
// Three tiles rotate through LDS: one is multiplied, the next has landed or is landing, the
// one after is being requested.  The epilogue of a finished tile (bias in fp32, ReLU,
// rounding, wave-private LDS transpose, row-contiguous non-temporal stores) is issued in
// pieces between the MFMAs of the next tile; two accumulator sets trade places.
// paper: Eq. "new_conv_H" with the dense K = KH*KW'*F*C_in of the expanded filter
// (Eq. "filter_construct"); Eq. "bias_construct"; Reconstruct step fused into the stores.
#include <hip/hip_runtime.h>

#include "launch.h"
#include "mfma_types.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <typename TR>
__device__ __forceinline__ unsigned pack2l(float a, float b);
template <>
__device__ __forceinline__ unsigned pack2l<F16Traits>(float a, float b) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 v = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(unsigned, v);
}
template <>
__device__ __forceinline__ unsigned pack2l<BF16Traits>(float a, float b) {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    b2 v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(unsigned, v);
}

__device__ __forceinline__ void wave_lds_sync_l() {
    // a wave's LDS instructions execute in issue order; only the compiler has to be held back
    __builtin_amdgcn_wave_barrier();
    asm volatile("" ::: "memory");
}

constexpr unsigned kOutOfRangeL = 0x80000000u;  // beyond any resource extent used here

struct LdsArgs {
    unsigned MT;          // number of 32-pixel M tiles
    FcDeal deal;          // how M tiles are dealt to the XCDs; deal.stride is the stride of a workgroup's tile walk
    int CQ;               // groups of 256 output columns (one workgroup each per tile)
    unsigned dW, dH;      // the walk stride of 32*stride pixels: folded columns and rows (mod the output height) moved
    int stepCol, wrapCol; // element column moved per step (dW*FC), and taken back when the folded column wraps (Wf_out*FC)
    unsigned stepOff, carryW, carryH;  // byte offset in x' moved per step, and the corrections of the two carries
    unsigned x_bytes;
};

// KHM = g.KH and QM = g.kwin / 8 (16-byte chunks of the K window per kh, even) exactly.
template <typename TR, int KHM, int QM, bool RELU>
__global__ void __launch_bounds__(256, 1)
conv_stream_lds_kernel(ConvGeom g, LdsArgs a, const typename TR::T *__restrict__ x, const u32x4 *__restrict__ wp,
                       const typename TR::T *__restrict__ bias, typename TR::T *__restrict__ y) {
    using Vec = typename TR::Vec;
    constexpr int NT = 2, COLS = 64;
    constexpr int KSM = QM / 2;                 // K-steps of 16 per kh
    constexpr int S = KHM * KSM;                // K-steps = staged fragments per tile
    constexpr int NLW = (S + 3) / 4;            // staging loads per wave and tile
    constexpr int FRAG = 1024;                  // one MFMA operand: 64 lanes x 16 bytes
    constexpr int STAGE = NLW * 4 * FRAG;       // fragments S .. 4*NLW-1 are never read
    constexpr int NSTAGE = 3;
    constexpr int kStores = 4;                  // 16-byte store instructions per wave and tile
    constexpr int PITCH = COLS * 2 + 16, SLAB = 32 * PITCH, CHUNKS = COLS / 8;
    __shared__ __attribute__((aligned(16))) unsigned char lds[NSTAGE * STAGE + 4 * SLAB];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, hf = lane >> 5;
    unsigned char *slab = lds + NSTAGE * STAGE + wave * SLAB;

    const unsigned part = blockIdx.x % a.deal.parts;
    const unsigned wgp = blockIdx.x / a.deal.parts;
    const int cq = (int)(wgp % (unsigned)a.CQ);
    const unsigned j0 = wgp / (unsigned)a.CQ;
    if (j0 >= a.deal.J) return;  // workgroup-uniform
    // Workgroup b runs on XCD b % parts; M tiles follow the workgroups in chunks (FcDeal).
    const unsigned t_first = fc_deal_first_tile(a.deal, part, j0);  // the workgroup's first tile
    const unsigned t_end = a.MT;
    const int n_lo = (cq * 4 + wave) * COLS;

    // ---- filter fragments for the whole K extent, resident for the kernel's lifetime ----
    Vec wf[S][NT];
#pragma unroll
    for (int idx = 0; idx < S; ++idx)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int kh = idx / KSM, q = 2 * (idx % KSM) + hf;
            const int n = n_lo + 32 * nt + r;
            const long long ci = g.compact ? fc_compact_chunk<8>(g, kh, q, n) : ((long long)kh * QM + q) * g.NCo + n;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (ci >= 0) v = wp[ci];  // structural zeros of the compact form
            wf[idx][nt] = __builtin_bit_cast(Vec, v);
        }
    // Keep the resident filter in the AGPR half of the register file (the MFMAs read their A operand from
    // there as well).  Built with the MFMA results in VGPRs (see the build script), the accumulators then
    // sit where the epilogue's VALU instructions read them directly, and nothing is copied between the halves.
#pragma unroll
    for (int idx = 0; idx < S; ++idx)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) asm volatile("" : "+a"(wf[idx][nt]));
    // The bias is added in fp32 when a finished tile is rounded (one add per output value, issued
    // between MFMAs): on this walk the matrix pipeline is the bottleneck, so it is not spent on a
    // rank-1 bias product as in the band-walk kernel.
    float bias_f[NT][16];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int n = n_lo + 32 * nt + 8 * (i / 4) + 4 * hf + (i % 4);  // the column of accumulator element i
            bias_f[nt][i] = g.has_bias ? (float)bias[n % g.Co] : 0.0f;
        }

    u32x4 xr;  // range-checked resource over x: out-of-range lanes deposit zeros (the zero padding)
    {
        const unsigned long long xa = (unsigned long long)x;
        xr[0] = __builtin_amdgcn_readfirstlane((unsigned)xa);
        xr[1] = __builtin_amdgcn_readfirstlane((unsigned)(xa >> 32) & 0xffffu);
        xr[2] = __builtin_amdgcn_readfirstlane(a.x_bytes);
        xr[3] = __builtin_amdgcn_readfirstlane(0x00020000u);
    }

    // per-lane constants of the row-wise store phase (as in the streaming kernel)
    constexpr int PASSES = (32 * CHUNKS + 63) / 64;
    static_assert(PASSES == kStores, "store count");
    int st_lds[PASSES];
    unsigned st_lin[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int idx = p * 64 + lane;
        const int row = idx / CHUNKS, ch = idx - row * CHUNKS;
        st_lds[p] = row * PITCH + ch * 16;
        st_lin[p] = 2u * ((unsigned)row * (unsigned)g.NCo + (unsigned)(n_lo + 8 * ch));
    }

    // ---- staging: fragment idx = 4*i + wave of a tile is requested by this wave's i-th load; lane
    //      (r, hf) asks for chunk q = 2*ks + hf of pixel r at row kh: exactly its MFMA operand ----
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)lds;
    // Walk state of this lane's pixel (pixel r of the tile requested next), kept incrementally: a
    // tile step is a constant number of pixels, so folded column, row and element offset move by
    // constants plus two carries; no multiplication or division inside the loop.
    unsigned p_m = t_first * 32u + (unsigned)r;  // pixel index
    unsigned p_wo = p_m % (unsigned)g.Wf_out, p_ho;     // folded column, output row
    unsigned p_off2;  // byte offset of x'[img][ho][wo] + the lane's chunk at e_min (may wrap below zero at the left edge)
    int p_col;        // element column of that chunk inside the input row
    {
        const unsigned rowid = p_m / (unsigned)g.Wf_out;
        p_ho = rowid % (unsigned)g.Hout;
        const unsigned img = rowid / (unsigned)g.Hout;
        p_col = (int)p_wo * g.FC + g.e_min + 8 * hf;
        p_off2 = 2u * (unsigned)((int)((img * (unsigned)g.H + p_ho) * (unsigned)g.in_row) + p_col);
    }
    int ld_stage = 0;
    unsigned ld_tile = t_first;
    int ld_vm = 0;         // this lane's pixel of the tile being requested exists
    unsigned ld_dst0 = 0;  // LDS address of this wave's first fragment in the tile's stage
    auto request_begin = [&]() {
        // false for tiles past the end of the walk: every lane out of range, zeros deposited, no traffic
        ld_vm = (int)(ld_tile < t_end) & (int)(p_m < (unsigned)g.M);
        ld_tile += a.deal.stride;
        ld_dst0 = lds_base + (unsigned)(ld_stage * STAGE + wave * FRAG);
        ld_stage = ld_stage + 1 == NSTAGE ? 0 : ld_stage + 1;
    };
    auto request_one = [&](int i) {
        const int idx = 4 * i + wave;  // wave-uniform
        const int kh = idx / KSM, ks = idx - kh * KSM;
        const int hi = (int)p_ho + (kh - g.pad_h), col = p_col + 16 * ks;
        const int ok = ld_vm & (int)(idx < S) & (int)((unsigned)hi < (unsigned)g.H) & (int)((unsigned)col < (unsigned)g.in_row);
        const unsigned voff = ok ? p_off2 + 2u * (unsigned)((kh - g.pad_h) * g.in_row + 16 * ks) : kOutOfRangeL;
        const unsigned dst = ld_dst0 + (unsigned)(4 * i * FRAG);
        asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" : : "s"(dst), "v"(voff), "s"(xr) : "memory");
    };
    auto request_end = [&]() {  // step the walk state to the next tile of this workgroup
        p_m += a.deal.stride * 32u;
        p_wo += a.dW;
        const bool c1 = p_wo >= (unsigned)g.Wf_out;
        p_wo -= c1 ? (unsigned)g.Wf_out : 0u;
        p_ho += a.dH + (c1 ? 1u : 0u);
        const bool c2 = p_ho >= (unsigned)g.Hout;
        p_ho -= c2 ? (unsigned)g.Hout : 0u;
        p_col += a.stepCol - (c1 ? a.wrapCol : 0);
        p_off2 += a.stepOff + (c1 ? a.carryW : 0u) + (c2 ? a.carryH : 0u);
    };

    // ---- epilogue of one tile, in pieces that are slotted between the MFMAs of the next tile ----
    // two accumulator sets trade places every tile: one is accumulated, the other (finished) is stored
    floatx16_t acc_a[NT], acc_b[NT];
    unsigned m0 = t_first * 32u;  // first pixel of the tile being accumulated
    unsigned d_m0 = 0;                   // ... of the finished tile
    int d_valid = 0;                             // 0: nothing finished yet, its stores are dropped
    __amdgpu_buffer_rsrc_t yr = __builtin_amdgcn_make_buffer_rsrc(y, 0, 0, 0x00020000);
    // Accumulator element 4*q + j of lane (r, hf) is column 8*q + 4*hf + j of pixel r: a lane holds 8-byte
    // pieces 16 bytes apart.  The two halves of the wave trade pieces (v_permlane32_swap: the upper 32
    // lanes of the first operand against the lower 32 lanes of the second), after which lane (r, 0) holds
    // columns 16*k .. 16*k+7 and lane (r, 1) columns 16*k+8 .. 16*k+15 of its pixel: one 16-byte LDS write
    // per lane, free of bank conflicts at this row pitch (8-byte writes collide two ways).
    auto epi_pack = [&](const floatx16_t (&done)[NT], int nt, int k) {
        u32x2 pk[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int q = 2 * k + h;
            const float *bq = &bias_f[nt][4 * q];
            pk[h] = u32x2{pack2l<TR>(done[nt][4 * q] + bq[0], done[nt][4 * q + 1] + bq[1]),
                          pack2l<TR>(done[nt][4 * q + 2] + bq[2], done[nt][4 * q + 3] + bq[3])};
            if (RELU) {
                typedef short s16x4 __attribute__((ext_vector_type(4)));
                const s16x4 z = {0, 0, 0, 0};
                pk[h] = __builtin_bit_cast(u32x2, __builtin_elementwise_max(__builtin_bit_cast(s16x4, pk[h]), z));
            }
        }
        const u32x2 s0 = __builtin_amdgcn_permlane32_swap(pk[0][0], pk[1][0], false, false);
        const u32x2 s1 = __builtin_amdgcn_permlane32_swap(pk[0][1], pk[1][1], false, false);
        const u32x4 v = {s0[0], s1[0], s0[1], s1[1]};
        *reinterpret_cast<u32x4 *>(slab + r * PITCH + (32 * nt + 16 * k + 8 * hf) * 2) = v;
    };
    auto epi_resource = [&]() {
        wave_lds_sync_l();
        // stored rows are exactly Wf_out*NCo long (checked by the launcher): y offset is m*NCo + n
        unsigned long long base_el = (unsigned long long)d_m0 * (unsigned)g.NCo;  // first element of the resource
        unsigned long long left_el = ((unsigned long long)g.M - d_m0) * (unsigned)g.NCo;  // elements to the end of y
        if (!d_valid) base_el = 0, left_el = 0;  // zero extent: every store is dropped
        const unsigned long long left_b = left_el * 2ull;
        yr = __builtin_amdgcn_make_buffer_rsrc(y + base_el, 0, (int)(left_b > 0x7fffffffull ? 0x7fffffffull : left_b), 0x00020000);
    };
    // the slab is read one piece ahead of its store, so that no store waits for an LDS read just issued
    u32x4 st_val[2];
    auto epi_read = [&](int p) { st_val[p & 1] = *reinterpret_cast<const u32x4 *>(slab + st_lds[p]); };
    auto epi_store = [&](int p) {
        if (p + 1 < kStores) epi_read(p + 1);
        __builtin_amdgcn_raw_buffer_store_b128(st_val[p & 1], yr, st_lin[p], 0, 2 /* nt */);  // rows past the end of y fall outside the resource
        if (p == kStores - 1) wave_lds_sync_l();
    };
    // piece number -> work: 4 pack-and-write pieces, the resource, the first read, 4 store(-and-read-next) pieces
    auto epi_piece = [&](const floatx16_t (&done)[NT], int k) {
        if (k < 4) epi_pack(done, k / 2, k % 2);
        else if (k == 4) epi_resource();
        else if (k == 5) epi_read(0);
        else if (k < 6 + kStores) epi_store(k - 6);
    };
    constexpr int kPieces = 6 + kStores;
    static_assert(S >= kPieces + 2 && S >= 4 * (NLW - 1) + 2, "the K loop is too short to hold the pieces");

    // Every tile's wait sees the same queue.  Each trip issues NLW loads (two tiles ahead) and
    // kStores stores (the tile before), so behind the last load of tile i there are at least the
    // NLW + kStores operations of the trip before this one.  Vector-memory operations complete in
    // issue order: "at most NLW + kStores outstanding" means tile i has reached LDS, while the
    // newest loads and stores stay in flight.  The prologue issues the same mix (its stores are
    // dropped), so the count holds for the first two tiles too.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // nothing the compiler tracks may be in flight
    request_begin();
#pragma unroll
    for (int i = 0; i < NLW; ++i) request_one(i);
    request_end();
    request_begin();
#pragma unroll
    for (int i = 0; i < NLW; ++i) request_one(i);
    request_end();
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc_a[nt][i] = acc_b[nt][i] = 0.0f;
#pragma unroll
    for (int k = 4; k < kPieces; ++k) epi_piece(acc_a, k);  // stores dropped: d_valid = 0

    int cur_stage = 0;
    // one tile: accumulate into `acc` while the finished tile in `done` is rounded and stored
    auto tile = [&](floatx16_t (&acc)[NT], const floatx16_t (&done)[NT]) {
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(NLW + kStores) : "memory");
        __builtin_amdgcn_s_barrier();  // the tile is in LDS for every wave; everyone is done with the stage requested next
        asm volatile("" ::: "memory");
        const unsigned char *sf = lds + cur_stage * STAGE + lane * 16;
        cur_stage = cur_stage + 1 == NSTAGE ? 0 : cur_stage + 1;
        auto frag = [&](int idx) { return *reinterpret_cast<const Vec *>(sf + idx * FRAG); };
        // fragments are read three K-steps ahead of their MFMAs; between the MFMA pairs go the
        // address arithmetic of the tile requested next (two tiles ahead), its staging loads, and
        // the pieces of the finished tile's epilogue
        Vec xb[4];
        xb[0] = frag(0);
        xb[1] = frag(1);
        xb[2] = frag(2);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[nt][i] = 0.0f;  // folded into the first MFMA's C operand
#pragma unroll
        for (int idx = 0; idx < S; ++idx) {
            if (idx + 3 < S) xb[(idx + 3) % 4] = frag(idx + 3);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[nt] = TR::mfma(wf[idx][nt], xb[idx % 4], acc[nt]);
            __builtin_amdgcn_sched_barrier(0);
            if (idx == 0) request_begin();
            if (idx % 4 == 1 && idx / 4 < NLW) request_one(idx / 4);
            if (idx == S - 1) request_end();
            if (idx >= 2 && idx - 2 < kPieces) epi_piece(done, idx - 2);
            __builtin_amdgcn_sched_barrier(0);
        }
        d_m0 = m0, d_valid = 1;  // this tile is finished; its epilogue rides along with the next one
        m0 += a.deal.stride * 32u;
    };
    bool last_in_a = false;
    for (unsigned mt = t_first; mt < t_end;) {
        tile(acc_a, acc_b);
        last_in_a = true;
        mt += a.deal.stride;
        if (mt >= t_end) break;
        tile(acc_b, acc_a);
        last_in_a = false;
        mt += a.deal.stride;
    }
    // the last tile's epilogue (dropped if the workgroup had no tile)
    if (last_in_a) {
#pragma unroll
        for (int k = 0; k < kPieces; ++k) epi_piece(acc_a, k);
    } else {
#pragma unroll
        for (int k = 0; k < kPieces; ++k) epi_piece(acc_b, k);
    }
    // drain the tiles requested past the end before the workgroup's LDS is released
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <typename TR, int KHM, int QM>
int launch_inst(const ConvGeom &g, const void *x, const void *wp, const void *bias, void *y, hipStream_t st) {
    using T = typename TR::T;
    LdsArgs a;
    a.MT = (unsigned)((g.M + 31) / 32);
    a.CQ = g.NCo / 256;
    FcDevice dev;
    if (int e = fc_device(&dev)) return e;
    const unsigned parts = a.MT >= 64 * dev.xcds ? dev.xcds : 1;
    a.deal = fc_make_deal(a.MT, parts, (dev.cus / parts) / (unsigned)a.CQ, g.KH, g.Wf_out);  // one workgroup per compute unit
    const long long J = a.deal.J;
    const long long S = (long long)a.deal.stride * 32, plane = (long long)g.Hout * g.Wf_out;
    const long long dI = S / plane;
    a.dH = (unsigned)((S % plane) / g.Wf_out);
    a.dW = (unsigned)((S % plane) % g.Wf_out);
    a.stepCol = (int)a.dW * g.FC;
    a.wrapCol = g.Wf_out * g.FC;
    // x'[img][ho][wo] sits at ((img*H + ho)*in_row + wo*FC) elements; a carry out of the folded column adds a
    // row and takes Wf_out columns back, a carry out of the row adds an image and takes Hout rows back
    a.stepOff = (unsigned)(2 * ((dI * g.H + a.dH) * g.in_row + (long long)a.dW * g.FC));
    a.carryW = (unsigned)(2 * ((long long)g.in_row - (long long)g.Wf_out * g.FC));
    a.carryH = (unsigned)(2 * ((long long)(g.H - g.Hout) * g.in_row));
    a.x_bytes = (unsigned)((long long)g.N * g.H * g.in_row * (long long)sizeof(T));
    const unsigned blocks = (unsigned)(J * a.CQ) * a.deal.parts;
    if (g.relu)
        conv_stream_lds_kernel<TR, KHM, QM, true><<<blocks, 256, 0, st>>>(g, a, (const T *)x, (const u32x4 *)wp, (const T *)bias, (T *)y);
    else
        conv_stream_lds_kernel<TR, KHM, QM, false><<<blocks, 256, 0, st>>>(g, a, (const T *)x, (const u32x4 *)wp, (const T *)bias, (T *)y);
    return (int)hipGetLastError();
}

template <typename TR>
int launch_any(const ConvGeom &g, const void *x, const void *wp, const void *bias, void *y, hipStream_t st) {
    const int Q = g.kwin / 8;
    if (g.KH == 3 && Q == 18) return launch_inst<TR, 3, 18>(g, x, wp, bias, y, st);
    return (int)hipErrorInvalidValue;
}

}  // namespace

int fc_launch_conv_stream_lds(foldconv_dtype_t dt, const ConvGeom &g, const void *x, const void *w_pack, const void *bias,
                              void *y, void *stream) {
    if (!fc_stream_lds_ok(g)) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    if (dt == FOLDCONV_F16) return launch_any<F16Traits>(g, x, w_pack, bias, y, st);
    if (dt == FOLDCONV_BF16) return launch_any<BF16Traits>(g, x, w_pack, bias, y, st);
    return (int)hipErrorInvalidValue;
}
