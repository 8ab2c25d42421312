// Wave-level pieces of the bf16 matrix-product loops that stream both operands through LDS in
// their natural layouts:
//   A operand  [rows][k], k contiguous   -> one 16-byte LDS read per fragment
//   W operand  [k][n],  n contiguous     -> two transposing 8-byte reads per fragment, so row-major
//                                           [K][N] weights feed the matrix cores untransposed
// A wave always owns a 64 x 96 tile (2 x 3 tiles of v_mfma_f32_32x32x16_bf16): every W fragment
// feeds two matrix instructions, which keeps the transposing reads (half the rate of 16-byte
// reads on this LDS) below the matrix pipe's time.
//
// LDS row strides: A rows are 16 bytes longer than their data (consecutive rows start 4 banks apart:
// a 16-lane group of 16-byte reads is conflict-free); W rows have a stride of 64 mod 256 bytes, so
// the four k-rows a 32-lane half of a transposing read touches (64 bytes each) tile the 64 banks.
#pragma once
#include "ago_dev.hpp"

namespace ago {

typedef __attribute__((address_space(3))) unsigned char lds_u8;
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 lds_read_a(const lds_u8* p) {
    typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
    return *(const lds_bf16x8*)p;
}
// p: this lane's address in k-row (k0 + lane-dependent row) of the W tile; stride: bytes per k-row
__device__ __forceinline__ bf16x8 lds_read_w(const lds_u8* p, int stride) {
    typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p + 4 * stride));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}
__device__ __forceinline__ void lds_write16(lds_u8* p, u32x4_t v) {
    typedef __attribute__((address_space(3))) u32x4_t lds_u32x4;
    *(lds_u32x4*)p = v;
}
__device__ __forceinline__ u32x4_t ldg16(const void* p) { return *reinterpret_cast<const u32x4_t*>(p); }

// Byte offset of this lane inside an A tile (row stride `stride` bytes) for the 32-row tile starting at
// row0 and the 16-deep k step starting at element k0.
__device__ __forceinline__ int a_frag_off(int lane, int row0, int k0, int stride) {
    return (row0 + (lane & 31)) * stride + (k0 + 8 * (lane >> 5)) * 2;
}
// Byte offset of this lane inside a W tile for the 32 columns starting at col0 and the 16-deep k step at
// k-row k0: lane group g = lane / 16 reads k-rows k0 + 8 (g / 2) + {0..3} (the second read +4) of
// columns col0 + 16 (g & 1) .. + 15; within a group, lanes 4 e .. 4 e + 3 address row e.
__device__ __forceinline__ int w_frag_off(int lane, int col0, int k0, int stride) {
    const int g = lane >> 4, s = lane & 15;
    return (k0 + 8 * (g >> 1) + (s >> 2)) * stride + (col0 + 16 * (g & 1)) * 2 + (s & 3) * 8;
}

struct Frag64x96 {
    bf16x8 a[2], w[3];
};

// acc (rows = A rows, lane = column) += A fragments x W fragments
__device__ __forceinline__ void mma_64x96(f32x16 (&acc)[2][3], const Frag64x96& f) {
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < 3; ++n) acc[m][n] = mfma32(f.a[m], f.w[n], acc[m][n]);
}

}  // namespace ago
