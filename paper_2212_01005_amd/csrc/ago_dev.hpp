// Device-side building blocks shared by the fused and the un-fused kernels:
// vector types, bf16 conversion, activations, and the wave-level MFMA tile loop.
//
// MFMA operand convention used everywhere (gfx950, wave64):
//   v_mfma_f32_32x32x16_bf16  D[32x32] += A[32x16] * B[16x32]
//     A: lane l holds row (l & 31), the 8 k-values of k-group (l >> 5)
//     B: lane l holds column (l & 31), the 8 k-values of k-group (l >> 5)
//     D: lane l holds column (l & 31); register r holds row 8*(r/4) + 4*(l>>5) + (r&3)
//   Both operands are therefore read from LDS tiles stored [row][k] with k contiguous
//   (one 16-byte read per operand).  Row-major [K][N] weights are transposed once
//   while they are staged into LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ago {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

enum Act : int { kNone = 0, kRelu = 1, kRelu6 = 2, kGeluTanh = 3 };

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
    return __builtin_bit_cast(float, (uint32_t)b << 16);
}
// round-to-nearest-even (the hardware conversion on gfx950)
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    return __builtin_bit_cast(uint16_t, (bf16_t)f);
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    bf16x2 v;
    v[0] = (bf16_t)lo;
    v[1] = (bf16_t)hi;
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float lo_bf16(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float hi_bf16(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }

// tanh-form GELU written as x * sigmoid(2u), u = sqrt(2/pi) (x + 0.044715 x^3):
// 1 / (1 + exp(-2u)) with exp2, exp(-2u) = 2^(x (a + b x^2)), a = -2 log2(e) sqrt(2/pi), b = 0.044715 a
// (the constants folded by hand: three multiply-adds ahead of the exponential instead of five)
__device__ __forceinline__ float gelu_tanh(float x) {
    constexpr float a = -2.302208198144325f, b = -0.1029432395800235f;
    const float e = __builtin_amdgcn_exp2f(x * fmaf(x * x, b, a));
    return x * __builtin_amdgcn_rcpf(1.0f + e);
}

template <int ACT>
__device__ __forceinline__ float apply_act(float v) {
    if constexpr (ACT == kRelu) return fmaxf(v, 0.0f);
    else if constexpr (ACT == kRelu6) return fminf(fmaxf(v, 0.0f), 6.0f);
    else if constexpr (ACT == kGeluTanh) return gelu_tanh(v);
    else return v;
}
__device__ __forceinline__ float apply_act_rt(float v, int act) {
    switch (act) {
        case kRelu: return fmaxf(v, 0.0f);
        case kRelu6: return fminf(fmaxf(v, 0.0f), 6.0f);
        case kGeluTanh: return gelu_tanh(v);
        default: return v;
    }
}

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row of the 32x32 accumulator tile held in register r of a lane in half `h` (= lane >> 5).
__device__ __forceinline__ int acc_row(int r, int h) { return 8 * (r >> 2) + 4 * h + (r & 3); }

// 16-byte LDS / global accessors
__device__ __forceinline__ bf16x8 ld_bf16x8(const void* p) { return *reinterpret_cast<const bf16x8*>(p); }
__device__ __forceinline__ uint4 ld_u4(const void* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ void st_u4(void* p, uint4 v) { *reinterpret_cast<uint4*>(p) = v; }

// Transpose a [8 k][4 n] block of bf16 held as 8 rows of uint2 (n0,n1 | n2,n3) into four
// 16-byte vectors, one per n, each holding the 8 k-values of that column.
__device__ __forceinline__ void transpose_8x4(const uint2 (&r)[8], uint4 (&out)[4]) {
    uint32_t o[4][4];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const uint2 e = r[2 * m], d = r[2 * m + 1];
        o[0][m] = (e.x & 0xffffu) | (d.x << 16);
        o[1][m] = (e.x >> 16) | (d.x & 0xffff0000u);
        o[2][m] = (e.y & 0xffffu) | (d.y << 16);
        o[3][m] = (e.y >> 16) | (d.y & 0xffff0000u);
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) out[t] = make_uint4(o[t][0], o[t][1], o[t][2], o[t][3]);
}

// One k16 step of a wave tile: acc[MT][NT] += A(rows) x B(rows)^T, both operands in LDS as
// [row][k] with `lda`/`ldb` bf16 elements per row.  a_base/b_base point at the wave's first
// row and the current k offset; lane addressing is done here.
template <int MT, int NT>
__device__ __forceinline__ void wave_mma_k16(f32x16 (&acc)[MT][NT], const bf16_t* a_base, int lda,
                                             const bf16_t* b_base, int ldb, int lane) {
    const int i = lane & 31, h = lane >> 5;
    bf16x8 af[MT], bfr[NT];
#pragma unroll
    for (int m = 0; m < MT; ++m) af[m] = ld_bf16x8(a_base + (m * 32 + i) * lda + 8 * h);
#pragma unroll
    for (int n = 0; n < NT; ++n) bfr[n] = ld_bf16x8(b_base + (n * 32 + i) * ldb + 8 * h);
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n) acc[m][n] = mfma32(af[m], bfr[n], acc[m][n]);
}

template <int MT, int NT>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[MT][NT]) {
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.0f;
}

}  // namespace ago
