// Element types and MFMA wrappers shared by the convolution kernels (gfx950).
//
// Operand convention used throughout: the MFMA "A" operand (32 rows) carries
// the filter, rows = output columns n; the "B" operand (32 columns) carries
// the folded input, columns = output pixels m.  Per lane l of the wave64:
//   16-bit types, v_mfma_f32_32x32x16_{f16,bf16}: A = w'[k0 + 8*(l/32) + j][n0 + l%32],
//     B = A_im2col[m0 + l%32][k0 + 8*(l/32) + j], j = 0..7 (both K-contiguous);
//   16-bit types in 8-byte chunks, v_mfma_f32_32x32x8_{f16,bf16} (F16HalfTraits, BF16HalfTraits): the same with
//     four K values per lane, k = k0 + 4*(l/32) + j, j = 0..3;
//   fp32, v_mfma_f32_32x32x2_f32: one element each, k = k0 + l/32 (the element-gather kernel), or
//     four (two) per lane used by four (two) MFMAs in turn (F32ChunkTraits, F32PairTraits: the streaming kernel).
// Accumulator register r (0..15) of lane l holds
//   D[n0 + 8*(r/4) + 4*(l/32) + r%4][m0 + l%32],
// i.e. four consecutive output channels of one pixel per register quad.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef short shortx4_t __attribute__((ext_vector_type(4)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));

struct F16Traits {
    using T = _Float16;
    using Vec = half8_t;
    static constexpr int kPerLane = 8;  // K elements per lane per MFMA
    static constexpr int kStep = 16;    // K elements per MFMA
    static __device__ __forceinline__ floatx16_t mfma(Vec a, Vec b, floatx16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    // the product when only element 0 of a and b is non-zero (the rank-1 bias term)
    static __device__ __forceinline__ floatx16_t mfma_k0(Vec a, Vec b, floatx16_t c) { return mfma(a, b, c); }
    static __device__ __forceinline__ T from_float(float v) { return (T)v; }
};

struct BF16Traits {
    using T = __bf16;
    using Vec = bf16x8_t;
    static constexpr int kPerLane = 8;
    static constexpr int kStep = 16;
    static __device__ __forceinline__ floatx16_t mfma(Vec a, Vec b, floatx16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ floatx16_t mfma_k0(Vec a, Vec b, floatx16_t c) { return mfma(a, b, c); }
    static __device__ __forceinline__ T from_float(float v) { return (T)v; }  // v_cvt_pk_bf16_f32: round to nearest even
};

// 16-bit types in 8-byte chunks of four K values, for layers whose F*C_in is a multiple of 4 but not of 8
// (the streaming kernel): a K-step of 8 is one v_mfma_f32_32x32x8.
struct F16HalfTraits {
    using T = _Float16;
    using Vec = half4_t;
    static constexpr int kPerLane = 4;
    static constexpr int kStep = 8;
    static __device__ __forceinline__ floatx16_t mfma(Vec a, Vec b, floatx16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x8f16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ floatx16_t mfma_k0(Vec a, Vec b, floatx16_t c) { return mfma(a, b, c); }
    static __device__ __forceinline__ T from_float(float v) { return (T)v; }
};

struct BF16HalfTraits {
    using T = __bf16;
    using Vec = bf16x4_t;
    static constexpr int kPerLane = 4;
    static constexpr int kStep = 8;
    static __device__ __forceinline__ floatx16_t mfma(Vec a, Vec b, floatx16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(shortx4_t, a), __builtin_bit_cast(shortx4_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ floatx16_t mfma_k0(Vec a, Vec b, floatx16_t c) { return mfma(a, b, c); }
    static __device__ __forceinline__ T from_float(float v) { return (T)v; }
};

// fp32 in 16-byte chunks, for the kernels that read four K-contiguous elements per lane: one K-step of 8 is
// four v_mfma_f32_32x32x2_f32, the j-th on element j of both operands (lane l: k = k0 + 4*(l/32) + j).
struct F32ChunkTraits {
    using T = float;
    using Vec = floatx4_t;
    static constexpr int kPerLane = 4;
    static constexpr int kStep = 8;
    static __device__ __forceinline__ floatx16_t mfma(Vec a, Vec b, floatx16_t c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[1], b[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[2], b[2], c, 0, 0, 0);
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a[3], b[3], c, 0, 0, 0);
    }
    // the product when only element 0 of a and b is non-zero (the rank-1 bias term): one MFMA instead of four
    static __device__ __forceinline__ floatx16_t mfma_k0(Vec a, Vec b, floatx16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0], c, 0, 0, 0);
    }
    static __device__ __forceinline__ T from_float(float v) { return v; }
};

// fp32 in 8-byte chunks of two K values: a K-step of 4 is two MFMAs.  Half the alignment loss of the 16-byte
// chunks on a narrow band (a 9-wide band costs 12 K values instead of 16), twice the load instructions.
struct F32PairTraits {
    using T = float;
    using Vec = floatx2_t;
    static constexpr int kPerLane = 2;
    static constexpr int kStep = 4;
    static __device__ __forceinline__ floatx16_t mfma(Vec a, Vec b, floatx16_t c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0], c, 0, 0, 0);
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a[1], b[1], c, 0, 0, 0);
    }
    static __device__ __forceinline__ floatx16_t mfma_k0(Vec a, Vec b, floatx16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0], c, 0, 0, 0);
    }
    static __device__ __forceinline__ T from_float(float v) { return v; }
};

struct F32Traits {
    using T = float;
    using Vec = float;
    static constexpr int kPerLane = 1;
    static constexpr int kStep = 2;
    static __device__ __forceinline__ floatx16_t mfma(Vec a, Vec b, floatx16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ T from_float(float v) { return v; }
};
