// Data-movement kernels of libfoldconv for gfx950: filter expansion, the
// fold copy, reconstruct (row-cropping copy), channel zero-padding for the
// reference path, and the re-ordering of the expanded filter into MFMA
// operand order.  All are pure moves of element bits (no arithmetic), so
// they are templated on the element's storage width only.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "launch.h"

namespace {

constexpr int kThreads = 256;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // a 16-byte lane access
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

inline unsigned blocks_for(long long work, int per_block, long long cap) {
    long long b = (work + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (unsigned)b;
}

// ---------------------------------------------------------------------------
// Structured filter expansion (paper: Eq. "filter_construct", Algorithm 1).
// One thread per element of w'; every element is written, zeros included, so
// the destination needs no prior clearing.  Gather form of the band:
//   w'[kh][dd][f*C+c][g*Co+co] = w[kh][F*(dd+d_min)+f-g+p][c][co]  if that tap
//   index is inside [0, KW), else 0.
// ---------------------------------------------------------------------------
// The source filter is addressed through four element strides, so the same
// kernel reads HWIO (strides KW*C*Co, C*Co, Co, 1) and OIHW with either image
// axis in the role of the folded one.
struct FilterStrides {
    long long kh, kw, c, co;
};

template <typename U>
__global__ void __launch_bounds__(kThreads)
expand_filter_kernel(const U *__restrict__ w, U *__restrict__ we, int KH, int KW, int C, int Co, int F,
                     int KWf, int d_min, int p, long long total, FilterStrides ws) {
    const long long stride = (long long)gridDim.x * kThreads;
    const int FC = F * C, FCo = F * Co;
    for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
        int nn = (int)(i % FCo);
        long long r = i / FCo;
        int cf = (int)(r % FC);
        r /= FC;
        int dd = (int)(r % KWf);
        int kh = (int)(r / KWf);
        int f = cf / C, c = cf - f * C;
        int g = nn / Co, co = nn - g * Co;
        int kw = F * (dd + d_min) + f - g + p;
        U v = 0;
        if (kw >= 0 && kw < KW) v = w[kh * ws.kh + kw * ws.kw + c * ws.c + co * ws.co];
        we[i] = v;
    }
}

// ---------------------------------------------------------------------------
// Straight copy, 16 bytes per lane, one access per lane: 4 KB per workgroup, and as many
// workgroups as there are 4 KB pieces.  The hardware dispatcher hands the pieces out in address
// order, which keeps the chip-wide read and write fronts compact; on MI355X this measured
// 6.6 TB/s against 5.4-6.0 TB/s for persistent grid-stride forms of the same copy.
// The width fold of a contiguous NHWC tensor is this copy
// (paper: Eq. "width_fold_def"; equal linear offsets before and after).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads)
copy16_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, long long n16) {
    const long long stride = (long long)gridDim.x * kThreads;
    for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

__global__ void __launch_bounds__(kThreads)
copy1_kernel(const unsigned char *__restrict__ src, unsigned char *__restrict__ dst, long long n) {
    const long long stride = (long long)gridDim.x * kThreads;
    for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// ---------------------------------------------------------------------------
// Reconstruct with a ragged tail (paper: Reconstruct step): destination rows
// hold the first `dst_row` units of source rows of `src_row` units.
// ---------------------------------------------------------------------------
template <typename V>
__global__ void __launch_bounds__(kThreads)
crop_rows_kernel(const V *__restrict__ src, V *__restrict__ dst, long long rows, int src_row, int dst_row) {
    const long long total = rows * dst_row;
    const long long stride = (long long)gridDim.x * kThreads;
    for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
        long long r = i / dst_row;
        int c = (int)(i - r * dst_row);
        dst[i] = src[r * src_row + c];
    }
}

// ---------------------------------------------------------------------------
// Channel zero-padding of the input for the reference path: one 16-byte
// chunk of x_pad per thread (C_pad is a multiple of 8, so a chunk never
// straddles pixels).  paper: the zero-padding alternative.
// ---------------------------------------------------------------------------
template <typename U>
__global__ void __launch_bounds__(kThreads)
pad_input_kernel(const U *__restrict__ x, U *__restrict__ xp, long long pixels, int C, int C_pad) {
    constexpr int EPC = 16 / sizeof(U);
    const int cpp = C_pad / EPC;  // chunks per pixel
    const long long total = pixels * cpp;
    const long long stride = (long long)gridDim.x * kThreads;
    for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
        long long pix = i / cpp;
        int c0 = (int)(i - pix * cpp) * EPC;
        U v[EPC];
#pragma unroll
        for (int j = 0; j < EPC; ++j) {
            int c = c0 + j;
            v[j] = c < C ? x[pix * C + c] : (U)0;
        }
        u32x4 out;
        __builtin_memcpy(&out, v, 16);
        reinterpret_cast<u32x4 *>(xp)[i] = out;
    }
}

template <typename U>
__global__ void __launch_bounds__(kThreads)
pad_filter_kernel(const U *__restrict__ w, U *__restrict__ wp, int taps, int C, int C_pad, int Co, int Co_pad) {
    const long long total = (long long)taps * C_pad * Co_pad;
    const long long stride = (long long)gridDim.x * kThreads;
    for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
        int co = (int)(i % Co_pad);
        long long r = i / Co_pad;
        int c = (int)(r % C_pad);
        long long t = r / C_pad;
        wp[i] = (c < C && co < Co) ? w[(t * C + c) * Co + co] : (U)0;
    }
}

// ---------------------------------------------------------------------------
// Expanded filter -> MFMA operand order, in chunks of E rows (ConvGeom.epc):
//   pack[kh][q][n][j] = w'[kh*kwin + E*q + j][n],  j = 0..E-1  (16 bytes, or 8 for E = 4 of a 16-bit type)
// so that one lane's E consecutive K values of one output column are a
// single load.
// ---------------------------------------------------------------------------
template <int N> struct ChunkOf;
template <> struct ChunkOf<16> { typedef u32x4 type; };
template <> struct ChunkOf<8> { typedef u32x2 type; };

template <typename U, int E>  // uint16_t: chunks of 8 or 4 rows; uint32_t (fp32): chunks of 4 or 2
__global__ void __launch_bounds__(kThreads)
pack_filter_kernel(const U *__restrict__ we, typename ChunkOf<E * sizeof(U)>::type *__restrict__ pack, int KH, int kwin, int NCo) {
    const int q_per_kh = kwin / E;
    const long long total = (long long)KH * q_per_kh * NCo;
    const long long stride = (long long)gridDim.x * kThreads;
    for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
        int n = (int)(i % NCo);
        long long r = i / NCo;  // kh*q_per_kh + q  ==  first filter row / E
        const U *srcp = we + (r * E) * NCo + n;
        U v[E];
#pragma unroll
        for (int j = 0; j < E; ++j) v[j] = srcp[(long long)j * NCo];
        typename ChunkOf<E * sizeof(U)>::type out;
        __builtin_memcpy(&out, v, sizeof(out));
        pack[i] = out;
    }
}

// ---------------------------------------------------------------------------
// Original filter -> compact MFMA operand storage (layout at fc_compact_chunk):
// one thread per chunk  cpk[ph][kh][j][co][0..E-1].  Only the non-zero
// blocks of the expanded filter exist in this form
// (paper: "Potential Optimizations for Sparsity", storing just the non-zero blocks).
// ---------------------------------------------------------------------------
template <typename U, int E>  // as pack_filter_kernel
__global__ void __launch_bounds__(kThreads)
compact_filter_kernel(const U *__restrict__ w, typename ChunkOf<E * sizeof(U)>::type *__restrict__ cpk, int KH,
                      int taps_c /* KW*C_in */, int Co, int cJ, int cgcd, long long total) {
    const long long stride = (long long)gridDim.x * kThreads;
    for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
        const int co = (int)(i % Co);
        long long r = i / Co;
        const int j = (int)(r % cJ);
        r /= cJ;
        const int kh = (int)(r % KH);
        const int ph = (int)(r / KH);
        U v[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int t = E * j + e - ph * cgcd;  // row of the kh-th KW*C_in x C_out tap matrix
            v[e] = (t >= 0 && t < taps_c) ? w[((long long)kh * taps_c + t) * Co + co] : (U)0;
        }
        typename ChunkOf<E * sizeof(U)>::type out;
        __builtin_memcpy(&out, v, sizeof(out));
        cpk[i] = out;
    }
}

// ---------------------------------------------------------------------------
// Channels-first front end (paper: Introduction, "height folding for NCHW
// format").  A spatial axis of an NCHW tensor is not adjacent to the channel
// axis in memory, so folding it into channels is a real re-index, not an alias.
// The folded tensors keep the channels-last form the MFMA kernels read,
//   x'[n][a][b'][f*C+c],  (a, F*b'+f) = (h, w) when W is folded, (w, h) when H is,
// which as bytes is the plan-space NHWC tensor [n][a][b][c].
//
// Input: one thread builds one 16-byte piece of x' from scalar reads of x;
// neighbouring lanes read neighbouring addresses of the same few channel planes, so the
// reads coalesce in the vector L1.
// ---------------------------------------------------------------------------
struct NchwMap {
    long long total;        // elements of the channels-last tensor
    int C, A, B;            // channels, plan-space rows and columns
    long long sC, sA, sB;   // element strides of (c, a, b) inside one NCHW image; image stride = C*A*B
};

template <typename U>
__global__ void __launch_bounds__(kThreads)
nchw_to_fold_kernel(const U *__restrict__ x, U *__restrict__ xf, NchwMap m, int vec) {
    constexpr int EPC = 16 / sizeof(U);
    const long long pieces = (m.total + EPC - 1) / EPC;
    const long long stride = (long long)gridDim.x * kThreads;
    const long long img = (long long)m.C * m.A * m.B;
    for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < pieces; i += stride) {
        long long e = i * EPC;
        int c = (int)(e % m.C);
        long long r = e / m.C;
        int b = (int)(r % m.B);
        r /= m.B;
        int a = (int)(r % m.A);
        long long n = r / m.A;
        U v[EPC];
#pragma unroll
        for (int j = 0; j < EPC; ++j) {
            v[j] = (e + j < m.total) ? x[n * img + c * m.sC + a * m.sA + b * m.sB] : (U)0;
            if (++c == m.C) {
                c = 0;
                if (++b == m.B) {
                    b = 0;
                    if (++a == m.A) { a = 0; ++n; }
                }
            }
        }
        if (vec && e + EPC <= m.total) {
            u32x4 out;
            __builtin_memcpy(&out, v, 16);
            // a plain store: the convolution that follows reads x' at once, out of the caches this leaves it in
            // (written non-temporally, the same launch took 12 us longer on the headline layer)
            reinterpret_cast<u32x4 *>(xf)[i] = out;
        } else {
#pragma unroll
            for (int j = 0; j < EPC; ++j)
                if (e + j < m.total) xf[e + j] = v[j];
        }
    }
}

// The same re-index for 16-bit tensors through LDS, 16 bytes per lane on both sides.  A workgroup takes
// TA consecutive plan rows a of one image, every b and c: in x' that is one contiguous run of TA*B*C
// elements; in x it is C*R runs of L contiguous elements (width fold: R = TA rows of L = B elements per
// channel plane; height fold: R = B image rows, of which the tile takes L = TA columns).  The runs go
// to LDS as [c][a][b] (width fold) or [c][b][a] (height fold) with an odd dword pitch, and each thread
// gathers the eight elements of a piece of x' from there.
struct NchwTile {
    int C, A, B;            // channels, plan-space rows and columns
    long long sC, sA, sB;   // element strides of (c, a, b) inside one NCHW image; one of sA, sB is 1
    int TA;                 // plan rows per tile (a multiple of 8 when sA == 1)
    int tiles_a;            // ceil(A / TA)
    int R, L;               // runs per channel and elements per run (see above)
    int la, lb, LC;         // LDS element strides of a, b and c
};

__global__ void __launch_bounds__(kThreads)
nchw_to_fold_tile_kernel(const uint16_t *__restrict__ x, uint16_t *__restrict__ xf, NchwTile m) {
    extern __shared__ __attribute__((aligned(16))) uint16_t fold_lds[];
    const int t = threadIdx.x;
    const long long n = blockIdx.x / m.tiles_a;
    const int a0 = (int)(blockIdx.x - n * m.tiles_a) * m.TA;
    const int ta = m.A - a0 < m.TA ? m.A - a0 : m.TA;  // rows of this tile
    const uint16_t *img = x + n * (long long)m.C * m.A * m.B;
    const bool w_fold = m.sB == 1;
    // ---- runs of x -> LDS, 16 bytes per load, four 4-byte LDS writes (the pitch is only 4-byte aligned) ----
    const int chunks_per_run = m.L >> 3;
    const int runs = m.C * m.R;
    for (int q = t; q < runs * chunks_per_run; q += kThreads) {
        const int run = q / chunks_per_run, k8 = (q - run * chunks_per_run) << 3;
        const int c = run / m.R, r = run - c * m.R;
        long long src;
        int dst;
        bool in;
        if (w_fold) {  // r = row of the tile, k8 = first column b of the chunk
            in = r < ta;
            src = c * m.sC + (long long)(a0 + r) * m.sA + k8;
            dst = c * m.LC + r * m.la + k8;
        } else {       // r = image row b, k8 = first row a of the chunk inside the tile
            in = k8 < ta;  // A is a multiple of 8: a chunk is whole or absent
            src = c * m.sC + (long long)r * m.sB + a0 + k8;
            dst = c * m.LC + r * m.lb + k8;
        }
        if (in) {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(img + src);
            unsigned *d = reinterpret_cast<unsigned *>(fold_lds + dst);
            d[0] = v[0]; d[1] = v[1]; d[2] = v[2]; d[3] = v[3];
        }
    }
    __syncthreads();
    // ---- pieces of x': eight consecutive (b, c) elements of the tile's contiguous run ----
    const int row = m.B * m.C;                 // elements per plan row of x', a multiple of 8
    const int pieces = ta * (row >> 3);
    u32x4 *out = reinterpret_cast<u32x4 *>(xf + ((n * m.A + a0) * (long long)row));
    for (int p = t; p < pieces; p += kThreads) {
        const int e = p << 3;
        int a = e / row;
        const int qq = e - a * row;
        int b = qq / m.C, c = qq - b * m.C;
        unsigned v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            v[j] = fold_lds[c * m.LC + a * m.la + b * m.lb];
            if (++c == m.C) {
                c = 0;
                if (++b == m.B) { b = 0; ++a; }
            }
        }
        u32x4 o = {v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16)};
        // a plain store: the convolution that follows reads x' at once, out of the caches this leaves it in
        out[p] = o;
    }
}

// Output: y'[n][a][b][co] (row pitch in b given, columns b >= B cropped: the ragged
// reconstruct) -> y[n][co][himg][wimg].  A workgroup moves a tile of 128 image columns x 64
// channels of one image row through LDS: 16-byte loads along co, eight 2-byte LDS reads per
// lane gather eight consecutive image columns of one channel, one 16-byte store along w
// (sixteen lanes write 256 consecutive bytes of a channel row: runs of 128 bytes cost a fifth more).
struct FoldToNchw {
    int Co, Hi, Wi;             // channels, image rows and columns of y
    long long sN, sH, sW;       // element strides of (n, himg, wimg) in y'
    int tiles_w, tiles_c;
    long long rows;             // N * Hi
};

constexpr int kTW = 128, kTC = 64;
constexpr int kTPitch = kTC * 2 + 4;  // bytes per LDS row; 33 dwords: the column gather hits distinct banks

__global__ void __launch_bounds__(kThreads)
fold_to_nchw_tile_kernel(const uint16_t *__restrict__ yf, uint16_t *__restrict__ y, FoldToNchw m) {
    __shared__ __attribute__((aligned(16))) unsigned char tile[kTW * kTPitch];
    const long long per_row = (long long)m.tiles_w * m.tiles_c;
    const long long total = m.rows * per_row;
    const int t = threadIdx.x;
    for (long long job = blockIdx.x; job < total; job += gridDim.x) {
        const long long row = job / per_row;           // n * Hi + himg
        const int rem = (int)(job - row * per_row);
        const int w0 = (rem / m.tiles_c) * kTW, c0 = (rem % m.tiles_c) * kTC;
        const long long n = row / m.Hi;
        const int hi = (int)(row - n * m.Hi);
        const uint16_t *src = yf + n * m.sN + hi * m.sH;
        // load: 128 pixels x 8 chunks of 8 channels
#pragma unroll
        for (int i = 0; i < (kTW * kTC / 8) / kThreads; ++i) {
            const int q = t + kThreads * i;
            const int px = q >> 3, ch = q & 7;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (w0 + px < m.Wi && c0 + 8 * ch < m.Co)
                v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + (w0 + px) * m.sW + c0 + 8 * ch));
            unsigned *dst = reinterpret_cast<unsigned *>(tile + px * kTPitch + 16 * ch);
            dst[0] = v[0]; dst[1] = v[1]; dst[2] = v[2]; dst[3] = v[3];
        }
        __syncthreads();
        // store: per channel, 16 chunks of 8 consecutive image columns
#pragma unroll
        for (int i = 0; i < (kTW * kTC / 8) / kThreads; ++i) {
            const int q = t + kThreads * i;
            const int wc = q % (kTW / 8), c = q / (kTW / 8);
            const int wbase = w0 + 8 * wc;
            if (c0 + c < m.Co && wbase < m.Wi) {
                uint16_t v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    v[k] = *reinterpret_cast<const uint16_t *>(tile + (8 * wc + k) * kTPitch + 2 * c);
                uint16_t *dst = y + ((n * m.Co + c0 + c) * m.Hi + hi) * (long long)m.Wi + wbase;
                if (wbase + 8 <= m.Wi) {
                    u32x4 out;
                    __builtin_memcpy(&out, v, 16);
                    __builtin_nontemporal_store(out, reinterpret_cast<u32x4 *>(dst));
                } else {
                    for (int k = 0; k < 8 && wbase + k < m.Wi; ++k) dst[k] = v[k];
                }
            }
        }
        __syncthreads();
    }
}

// Any element size and alignment: one thread per element of y, writes coalesced along w.
template <typename U>
__global__ void __launch_bounds__(kThreads)
fold_to_nchw_elem_kernel(const U *__restrict__ yf, U *__restrict__ y, FoldToNchw m) {
    const long long total = m.rows * m.Co * m.Wi;
    const long long stride = (long long)gridDim.x * kThreads;
    for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
        const int wi = (int)(i % m.Wi);
        long long r = i / m.Wi;
        const int hi = (int)(r % m.Hi);
        r /= m.Hi;
        const int co = (int)(r % m.Co);
        const long long n = r / m.Co;
        y[i] = yf[n * m.sN + hi * m.sH + wi * m.sW + co];
    }
}

inline int last_error() { return (int)hipGetLastError(); }

}  // namespace

int fc_launch_expand(const foldconv_plan_s *p, const void *w, void *w_exp, int oihw, void *stream) {
    const foldconv_shapes_t &s = p->s;
    const long long total = s.gemm_K * s.gemm_N;
    const unsigned grid = blocks_for(total, kThreads, 1 << 16);
    hipStream_t st = (hipStream_t)stream;
    FilterStrides ws;
    if (!oihw) {
        ws.co = 1; ws.c = s.C_out; ws.kw = (long long)s.C_in * s.C_out; ws.kh = ws.kw * s.KW;
    } else {
        // w[Co][C][KH_img][KW_img]; the plan's (KH, KW) are the image's (KH, KW), or (KW, KH) when H is folded
        const long long taps = (long long)s.KH * s.KW;
        ws.co = (long long)s.C_in * taps; ws.c = taps;
        if (p->fold_axis == FOLDCONV_FOLD_H) { ws.kh = 1; ws.kw = s.KH; }
        else { ws.kh = s.KW; ws.kw = 1; }
    }
    if (s.elem_bytes == 2)
        expand_filter_kernel<uint16_t><<<grid, kThreads, 0, st>>>((const uint16_t *)w, (uint16_t *)w_exp, s.KH, s.KW,
                                                                   s.C_in, s.C_out, s.F, s.KW_fold, s.d_min, s.pad_w, total, ws);
    else
        expand_filter_kernel<uint32_t><<<grid, kThreads, 0, st>>>((const uint32_t *)w, (uint32_t *)w_exp, s.KH, s.KW,
                                                                   s.C_in, s.C_out, s.F, s.KW_fold, s.d_min, s.pad_w, total, ws);
    return last_error();
}

int fc_launch_copy(const void *src, void *dst, size_t bytes, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    if (bytes == 0) return 0;
    if (((uintptr_t)src | (uintptr_t)dst) % 16 == 0) {
        const long long n16 = (long long)(bytes / 16);
        if (n16 > 0) {
            const unsigned grid = blocks_for(n16, kThreads, 1 << 22);
            copy16_kernel<<<grid, kThreads, 0, st>>>((const u32x4 *)src, (u32x4 *)dst, n16);
        }
        const size_t tail = bytes % 16;
        if (tail)
            copy1_kernel<<<1, kThreads, 0, st>>>((const unsigned char *)src + (bytes - tail),
                                                 (unsigned char *)dst + (bytes - tail), (long long)tail);
    } else {
        copy1_kernel<<<blocks_for((long long)bytes, kThreads, 1 << 16), kThreads, 0, st>>>(
            (const unsigned char *)src, (unsigned char *)dst, (long long)bytes);
    }
    return last_error();
}

int fc_launch_unfold(const foldconv_plan_s *p, const void *y_fold, void *y, void *stream) {
    const foldconv_shapes_t &s = p->s;
    hipStream_t st = (hipStream_t)stream;
    const long long rows = (long long)s.N * s.H_out;
    const long long src_row_b = (long long)s.W_out_fold * s.Co_fold * s.elem_bytes;
    const long long dst_row_b = (long long)s.W_out * s.C_out * s.elem_bytes;
    if (src_row_b % 16 == 0 && dst_row_b % 16 == 0 && ((uintptr_t)y_fold | (uintptr_t)y) % 16 == 0) {
        const unsigned grid = blocks_for(rows * (dst_row_b / 16), kThreads, 1 << 22);
        crop_rows_kernel<u32x4><<<grid, kThreads, 0, st>>>((const u32x4 *)y_fold, (u32x4 *)y, rows,
                                                           (int)(src_row_b / 16), (int)(dst_row_b / 16));
    } else if (s.elem_bytes == 2) {
        const unsigned grid = blocks_for(rows * (dst_row_b / 2), kThreads, 1 << 22);
        crop_rows_kernel<uint16_t><<<grid, kThreads, 0, st>>>((const uint16_t *)y_fold, (uint16_t *)y, rows,
                                                              (int)(src_row_b / 2), (int)(dst_row_b / 2));
    } else {
        const unsigned grid = blocks_for(rows * (dst_row_b / 4), kThreads, 1 << 22);
        crop_rows_kernel<uint32_t><<<grid, kThreads, 0, st>>>((const uint32_t *)y_fold, (uint32_t *)y, rows,
                                                              (int)(src_row_b / 4), (int)(dst_row_b / 4));
    }
    return last_error();
}

int fc_launch_pad_input(const foldconv_plan_s *p, const void *x, void *x_pad, void *stream) {
    const foldconv_shapes_t &s = p->s;
    hipStream_t st = (hipStream_t)stream;
    const long long pixels = (long long)s.N * s.H * s.W;
    const long long chunks = pixels * s.C_pad * s.elem_bytes / 16;
    const unsigned grid = blocks_for(chunks, kThreads, 1 << 22);
    if (s.elem_bytes == 2)
        pad_input_kernel<uint16_t><<<grid, kThreads, 0, st>>>((const uint16_t *)x, (uint16_t *)x_pad, pixels, s.C_in, s.C_pad);
    else
        pad_input_kernel<uint32_t><<<grid, kThreads, 0, st>>>((const uint32_t *)x, (uint32_t *)x_pad, pixels, s.C_in, s.C_pad);
    return last_error();
}

int fc_launch_pad_filter(const foldconv_plan_s *p, const void *w, void *w_pad, void *stream) {
    const foldconv_shapes_t &s = p->s;
    hipStream_t st = (hipStream_t)stream;
    const int taps = s.KH * s.KW;
    const long long total = (long long)taps * s.C_pad * s.C_out_pad;
    const unsigned grid = blocks_for(total, kThreads, 1 << 16);
    if (s.elem_bytes == 2)
        pad_filter_kernel<uint16_t><<<grid, kThreads, 0, st>>>((const uint16_t *)w, (uint16_t *)w_pad, taps, s.C_in, s.C_pad, s.C_out, s.C_out_pad);
    else
        pad_filter_kernel<uint32_t><<<grid, kThreads, 0, st>>>((const uint32_t *)w, (uint32_t *)w_pad, taps, s.C_in, s.C_pad, s.C_out, s.C_out_pad);
    return last_error();
}

// bias [C_out] -> [C_out_pad], zeros appended (the filter padding with one tap and one input channel)
int fc_launch_pad_bias(const foldconv_plan_s *p, const void *b, void *b_pad, void *stream) {
    const foldconv_shapes_t &s = p->s;
    hipStream_t st = (hipStream_t)stream;
    if (s.elem_bytes == 2)
        pad_filter_kernel<uint16_t><<<1, kThreads, 0, st>>>((const uint16_t *)b, (uint16_t *)b_pad, 1, 1, 1, s.C_out, s.C_out_pad);
    else
        pad_filter_kernel<uint32_t><<<1, kThreads, 0, st>>>((const uint32_t *)b, (uint32_t *)b_pad, 1, 1, 1, s.C_out, s.C_out_pad);
    return last_error();
}

// y_pad [pixels][C_out_pad] -> y [pixels][C_out]
int fc_launch_crop_channels(const foldconv_plan_s *p, const void *y_pad, void *y, void *stream) {
    const foldconv_shapes_t &s = p->s;
    hipStream_t st = (hipStream_t)stream;
    const long long pixels = (long long)s.N * s.H_out * s.W_out;
    const unsigned grid = blocks_for(pixels * s.C_out, kThreads, 1 << 22);
    if (s.elem_bytes == 2)
        crop_rows_kernel<uint16_t><<<grid, kThreads, 0, st>>>((const uint16_t *)y_pad, (uint16_t *)y, pixels, s.C_out_pad, s.C_out);
    else
        crop_rows_kernel<uint32_t><<<grid, kThreads, 0, st>>>((const uint32_t *)y_pad, (uint32_t *)y, pixels, s.C_out_pad, s.C_out);
    return last_error();
}

// the operand chunks the packers write: 8 or 4 elements of a 16-bit type, 4 or 2 of fp32
static bool chunk_ok(const ConvGeom &g) { return (g.eb == 2 && (g.epc == 8 || g.epc == 4)) || (g.eb == 4 && (g.epc == 4 || g.epc == 2)); }

int fc_launch_pack(const ConvGeom &g, int elem_bytes, const void *w_exp, void *w_pack, void *stream) {
    if (elem_bytes != g.eb || !chunk_ok(g) || g.kwin % g.epc != 0) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    const long long total = (long long)g.KH * (g.kwin / g.epc) * g.NCo;
    const unsigned grid = blocks_for(total, kThreads, 1 << 16);
    if (elem_bytes == 2 && g.epc == 8)
        pack_filter_kernel<uint16_t, 8><<<grid, kThreads, 0, st>>>((const uint16_t *)w_exp, (u32x4 *)w_pack, g.KH, g.kwin, g.NCo);
    else if (elem_bytes == 2)
        pack_filter_kernel<uint16_t, 4><<<grid, kThreads, 0, st>>>((const uint16_t *)w_exp, (u32x2 *)w_pack, g.KH, g.kwin, g.NCo);
    else if (g.epc == 4)
        pack_filter_kernel<uint32_t, 4><<<grid, kThreads, 0, st>>>((const uint32_t *)w_exp, (u32x4 *)w_pack, g.KH, g.kwin, g.NCo);
    else
        pack_filter_kernel<uint32_t, 2><<<grid, kThreads, 0, st>>>((const uint32_t *)w_exp, (u32x2 *)w_pack, g.KH, g.kwin, g.NCo);
    return last_error();
}

int fc_launch_compact(const ConvGeom &g, int elem_bytes, const void *w, void *w_compact, void *stream) {
    if (elem_bytes != g.eb || !chunk_ok(g) || g.FC % g.epc != 0) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    const long long total = (long long)fc_compact_phases(g) * g.KH * g.cJ * g.Co;
    const unsigned grid = blocks_for(total, kThreads, 1 << 16);
    if (elem_bytes == 2 && g.epc == 8)
        compact_filter_kernel<uint16_t, 8><<<grid, kThreads, 0, st>>>((const uint16_t *)w, (u32x4 *)w_compact, g.KH,
                                                                      g.KW * g.C, g.Co, g.cJ, g.cgcd, total);
    else if (elem_bytes == 2)
        compact_filter_kernel<uint16_t, 4><<<grid, kThreads, 0, st>>>((const uint16_t *)w, (u32x2 *)w_compact, g.KH,
                                                                      g.KW * g.C, g.Co, g.cJ, g.cgcd, total);
    else if (g.epc == 4)
        compact_filter_kernel<uint32_t, 4><<<grid, kThreads, 0, st>>>((const uint32_t *)w, (u32x4 *)w_compact, g.KH,
                                                                      g.KW * g.C, g.Co, g.cJ, g.cgcd, total);
    else
        compact_filter_kernel<uint32_t, 2><<<grid, kThreads, 0, st>>>((const uint32_t *)w, (u32x2 *)w_compact, g.KH,
                                                                      g.KW * g.C, g.Co, g.cJ, g.cgcd, total);
    return last_error();
}

int fc_launch_fold_nchw(const foldconv_plan_s *p, const void *x, void *x_fold, void *stream) {
    const foldconv_shapes_t &s = p->s;
    hipStream_t st = (hipStream_t)stream;
    NchwMap m;
    m.C = s.C_in; m.A = s.H; m.B = s.W;
    m.total = (long long)s.N * s.H * s.W * s.C_in;
    m.sC = (long long)s.H * s.W;
    if (p->fold_axis == FOLDCONV_FOLD_H) { m.sA = 1; m.sB = s.H; }   // image is [C][W_plan = H_img][H_plan = W_img]
    else { m.sA = s.W; m.sB = 1; }
    // 16-bit tensors whose rows split into whole 16-byte pieces on both sides go through LDS
    if (s.elem_bytes == 2 && ((uintptr_t)x | (uintptr_t)x_fold) % 16 == 0 && ((long long)m.B * m.C) % 8 == 0 &&
        (m.sB == 1 ? m.B % 8 == 0 : m.A % 8 == 0)) {
        NchwTile tl;
        tl.C = m.C; tl.A = m.A; tl.B = m.B; tl.sC = m.sC; tl.sA = m.sA; tl.sB = m.sB;
        const bool w_fold = m.sB == 1;
        // plan rows per tile: 16 rows of a width fold, 32 columns of a height fold (64-byte runs of x),
        // fewer while the tile does not fit 64 KB of LDS
        int TA = w_fold ? 16 : 32;
        auto lds_bytes = [&](int ta) {
            const long long pitch = (w_fold ? m.B : ta) + 2;  // elements; an odd number of dwords
            return 2ll * m.C * (w_fold ? ta : m.B) * pitch;
        };
        while (TA > (w_fold ? 1 : 8) && lds_bytes(TA) > 65536) TA /= 2;
        if (lds_bytes(TA) <= 65536 && (long long)s.N * ((m.A + TA - 1) / TA) < (1ll << 31)) {
            tl.TA = TA;
            tl.tiles_a = (m.A + TA - 1) / TA;
            const int pitch = (w_fold ? m.B : TA) + 2;
            if (w_fold) { tl.R = TA; tl.L = m.B; tl.la = pitch; tl.lb = 1; tl.LC = TA * pitch; }
            else { tl.R = m.B; tl.L = TA; tl.la = 1; tl.lb = pitch; tl.LC = m.B * pitch; }
            nchw_to_fold_tile_kernel<<<(unsigned)(s.N * tl.tiles_a), kThreads, (size_t)lds_bytes(TA), st>>>(
                (const uint16_t *)x, (uint16_t *)x_fold, tl);
            return last_error();
        }
    }
    const int vec = ((uintptr_t)x_fold % 16 == 0) ? 1 : 0;
    const long long pieces = (m.total * s.elem_bytes + 15) / 16;
    const unsigned grid = blocks_for(pieces, kThreads, 1 << 22);
    if (s.elem_bytes == 2)
        nchw_to_fold_kernel<uint16_t><<<grid, kThreads, 0, st>>>((const uint16_t *)x, (uint16_t *)x_fold, m, vec);
    else
        nchw_to_fold_kernel<uint32_t><<<grid, kThreads, 0, st>>>((const uint32_t *)x, (uint32_t *)x_fold, m, vec);
    return last_error();
}

int fc_launch_unfold_nchw(const foldconv_plan_s *p, const void *y_fold, void *y, void *stream) {
    const foldconv_shapes_t &s = p->s;
    hipStream_t st = (hipStream_t)stream;
    FoldToNchw m;
    const long long pitch_b = (long long)s.W_out_fold * s.Co_fold;  // elements per plan-space row of y'
    m.Co = s.C_out;
    m.sN = (long long)s.H_out * pitch_b;
    if (p->fold_axis == FOLDCONV_FOLD_H) {
        m.Hi = s.W_out; m.Wi = s.H_out;  // image rows run along the plan's folded axis
        m.sH = s.C_out; m.sW = pitch_b;
    } else {
        m.Hi = s.H_out; m.Wi = s.W_out;
        m.sH = pitch_b; m.sW = s.C_out;
    }
    m.rows = (long long)s.N * m.Hi;
    m.tiles_w = (m.Wi + kTW - 1) / kTW;
    m.tiles_c = (m.Co + kTC - 1) / kTC;
    const bool tiled = s.elem_bytes == 2 && s.C_out % 8 == 0 && m.Wi % 8 == 0 &&
                       ((uintptr_t)y_fold | (uintptr_t)y) % 16 == 0;
    if (tiled) {
        const unsigned grid = blocks_for(m.rows * m.tiles_w * m.tiles_c, 1, 1 << 22);
        fold_to_nchw_tile_kernel<<<grid, kThreads, 0, st>>>((const uint16_t *)y_fold, (uint16_t *)y, m);
    } else {
        const unsigned grid = blocks_for(m.rows * m.Co * m.Wi, kThreads, 1 << 22);
        if (s.elem_bytes == 2)
            fold_to_nchw_elem_kernel<uint16_t><<<grid, kThreads, 0, st>>>((const uint16_t *)y_fold, (uint16_t *)y, m);
        else
            fold_to_nchw_elem_kernel<uint32_t><<<grid, kThreads, 0, st>>>((const uint32_t *)y_fold, (uint32_t *)y, m);
    }
    return last_error();
}
