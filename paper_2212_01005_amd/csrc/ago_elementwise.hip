// Un-fused simple operators (one memory pass each): bias+activation, add+activation,
// scale, row softmax.  HBM-bound: 16-byte loads and stores, grid-stride loops.
#include "ago_dev.hpp"
#include "ago_launch.hpp"

namespace ago {

template <bool BF16>
struct Vec8 {  // 8 consecutive elements as fp32
    float v[8];
    __device__ __forceinline__ void load(const void* base, long idx8) {
        if constexpr (BF16) {
            const uint4 u = reinterpret_cast<const uint4*>(base)[idx8];
            v[0] = lo_bf16(u.x); v[1] = hi_bf16(u.x); v[2] = lo_bf16(u.y); v[3] = hi_bf16(u.y);
            v[4] = lo_bf16(u.z); v[5] = hi_bf16(u.z); v[6] = lo_bf16(u.w); v[7] = hi_bf16(u.w);
        } else {
            const float4 a = reinterpret_cast<const float4*>(base)[2 * idx8];
            const float4 b = reinterpret_cast<const float4*>(base)[2 * idx8 + 1];
            v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        }
    }
    __device__ __forceinline__ void store(void* base, long idx8) const {
        if constexpr (BF16) {
            reinterpret_cast<uint4*>(base)[idx8] = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]),
                                                              pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
        } else {
            reinterpret_cast<float4*>(base)[2 * idx8] = make_float4(v[0], v[1], v[2], v[3]);
            reinterpret_cast<float4*>(base)[2 * idx8 + 1] = make_float4(v[4], v[5], v[6], v[7]);
        }
    }
};

template <bool BF16>
__global__ __launch_bounds__(256) void bias_act_kernel(const void* x, const float* __restrict__ bias,
                                                       void* y, long n8, int C8, int act) {
    for (long i = blockIdx.x * 256L + threadIdx.x; i < n8; i += (long)gridDim.x * 256) {
        Vec8<BF16> v;
        v.load(x, i);
        const int c = (int)(i % C8) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) v.v[e] = apply_act_rt(v.v[e] + (bias ? bias[c + e] : 0.0f), act);
        v.store(y, i);
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void add_act_kernel(const void* a, const void* b, void* y, long n8,
                                                      int act) {
    for (long i = blockIdx.x * 256L + threadIdx.x; i < n8; i += (long)gridDim.x * 256) {
        Vec8<BF16> u, w;
        u.load(a, i);
        w.load(b, i);
#pragma unroll
        for (int e = 0; e < 8; ++e) u.v[e] = apply_act_rt(u.v[e] + w.v[e], act);
        u.store(y, i);
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void scale_kernel(const void* x, void* y, long n8, float alpha) {
    for (long i = blockIdx.x * 256L + threadIdx.x; i < n8; i += (long)gridDim.x * 256) {
        Vec8<BF16> u;
        u.load(x, i);
#pragma unroll
        for (int e = 0; e < 8; ++e) u.v[e] *= alpha;
        u.store(y, i);
    }
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// One wave per row; the row (cols <= 4096) lives in registers: 8 elements per lane per pass.
template <bool BF16, bool OUT_BF16>
__global__ __launch_bounds__(256) void softmax_rows_kernel(const void* x, void* y, long rows, int cols, int ld) {
    constexpr int MAXP = 8;  // 8 passes x 64 lanes x 8 elements = 4096 columns
    const int lane = threadIdx.x & 63;
    const long row = blockIdx.x * 4L + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int c8 = ld / 8;          // rows are ld elements apart; columns cols .. ld - 1 count as -inf and are written as 0
    const long base8 = row * c8;
    Vec8<BF16> v[MAXP];
    float m = -INFINITY;
#pragma unroll
    for (int p = 0; p < MAXP; ++p) {
        const int idx = p * 64 + lane;
        if (idx < c8) {
            v[p].load(x, base8 + idx);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (8 * idx + e >= cols) v[p].v[e] = -INFINITY;
                m = fmaxf(m, v[p].v[e]);
            }
        }
    }
    m = wave_max(m);
    float s = 0.0f;
#pragma unroll
    for (int p = 0; p < MAXP; ++p) {
        const int idx = p * 64 + lane;
        if (idx < c8) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                v[p].v[e] = __builtin_amdgcn_exp2f((v[p].v[e] - m) * 1.4426950408889634f);
                s += v[p].v[e];
            }
        }
    }
    s = wave_sum(s);
    const float inv = 1.0f / s;
#pragma unroll
    for (int p = 0; p < MAXP; ++p) {
        const int idx = p * 64 + lane;
        if (idx < c8) {
            Vec8<OUT_BF16> w;
#pragma unroll
            for (int e = 0; e < 8; ++e) w.v[e] = v[p].v[e] * inv;
            w.store(y, base8 + idx);
        }
    }
}

static inline int grid_for(long n8) {
    long g = (n8 + 255) / 256;
    return (int)(g < 1 ? 1 : (g > 2048 ? 2048 : g));
}

hipError_t bias_act(const void* x, const float* bias, void* y, long P, int C, int act, bool bf16,
                    hipStream_t s) {
    const long n8 = P * C / 8;
    if (bf16) hipLaunchKernelGGL(bias_act_kernel<true>, dim3(grid_for(n8)), dim3(256), 0, s, x, bias, y, n8, C / 8, act);
    else hipLaunchKernelGGL(bias_act_kernel<false>, dim3(grid_for(n8)), dim3(256), 0, s, x, bias, y, n8, C / 8, act);
    return hipGetLastError();
}

hipError_t add_act(const void* a, const void* b, void* y, long n, int act, bool bf16, hipStream_t s) {
    const long n8 = n / 8;
    if (bf16) hipLaunchKernelGGL(add_act_kernel<true>, dim3(grid_for(n8)), dim3(256), 0, s, a, b, y, n8, act);
    else hipLaunchKernelGGL(add_act_kernel<false>, dim3(grid_for(n8)), dim3(256), 0, s, a, b, y, n8, act);
    return hipGetLastError();
}

hipError_t scale(const void* x, void* y, long n, float alpha, bool bf16, hipStream_t s) {
    const long n8 = n / 8;
    if (bf16) hipLaunchKernelGGL(scale_kernel<true>, dim3(grid_for(n8)), dim3(256), 0, s, x, y, n8, alpha);
    else hipLaunchKernelGGL(scale_kernel<false>, dim3(grid_for(n8)), dim3(256), 0, s, x, y, n8, alpha);
    return hipGetLastError();
}

hipError_t softmax_rows(const void* x, void* y, long rows, int cols, bool in_bf16, bool out_bf16,
                        hipStream_t s, int ld) {
    if (ld == 0) ld = cols;
    const unsigned grid = (unsigned)((rows + 3) / 4);
    if (in_bf16 && out_bf16) hipLaunchKernelGGL((softmax_rows_kernel<true, true>), dim3(grid), dim3(256), 0, s, x, y, rows, cols, ld);
    else if (!in_bf16 && out_bf16) hipLaunchKernelGGL((softmax_rows_kernel<false, true>), dim3(grid), dim3(256), 0, s, x, y, rows, cols, ld);
    else if (!in_bf16 && !out_bf16) hipLaunchKernelGGL((softmax_rows_kernel<false, false>), dim3(grid), dim3(256), 0, s, x, y, rows, cols, ld);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ago
