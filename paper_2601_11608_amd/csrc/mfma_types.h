// Element types and MFMA wrappers shared by the convolution kernels (gfx950).
//
// Operand convention used throughout: the MFMA "A" operand (32 rows) carries
// the filter, rows = output columns n; the "B" operand (32 columns) carries
// the folded input, columns = output pixels m.  Per lane l of the wave64:
//   16-bit types, v_mfma_f32_32x32x16_{f16,bf16}: A = w'[k0 + 8*(l/32) + j][n0 + l%32],
//     B = A_im2col[m0 + l%32][k0 + 8*(l/32) + j], j = 0..7 (both K-contiguous);
//   fp32, v_mfma_f32_32x32x2_f32: one element each, k = k0 + l/32.
// Accumulator register r (0..15) of lane l holds
//   D[n0 + 8*(r/4) + 4*(l/32) + r%4][m0 + l%32],
// i.e. four consecutive output channels of one pixel per register quad.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

struct F16Traits {
    using T = _Float16;
    using Vec = half8_t;
    static constexpr int kPerLane = 8;  // K elements per lane per MFMA
    static constexpr int kStep = 16;    // K elements per MFMA
    static __device__ __forceinline__ floatx16_t mfma(Vec a, Vec b, floatx16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
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
    static __device__ __forceinline__ T from_float(float v) { return (T)v; }  // v_cvt_pk_bf16_f32: round to nearest even
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
