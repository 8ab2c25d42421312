// Un-fused matrix products (one complex operator per kernel, optional epilogue):
// ago_gemm / ago_conv1x1 (bf16 and fp32), ago_bmm_nt, ago_bmm_nn.
#include "ago_dev.hpp"
#include "ago_launch.hpp"

namespace ago {

// ---------------------------------------------------------------------------------------
// bf16 GEMM, fp32 accumulation.  C[M][N] = act(alpha * A[M][K] * B + bias)
//   B_NK = false: B is [K][N] row-major (weights);  B_NK = true: B is [N][K] (bmm_nt).
// Workgroup = 256 threads = WM x WN waves, tile BM x BN, K step 64, double-buffered LDS.
// grid = (ceil(N/BN), ceil(M/BM), batch)
// ---------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, bool B_NK, bool OUT_F32>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, const float* __restrict__ bias,
    const bf16_t* __restrict__ R, void* __restrict__ Cv, int M, int K, int N, int act, float alpha,
    long strideA, long strideB, long strideC) {
    constexpr int BK = 64, LD = BK + 8;
    constexpr int MT = BM / WM / 32, NT = BN / WN / 32;
    constexpr int A_CH = BM * BK / 8 / 256;          // 16-byte chunks of A per thread
    constexpr int BN_CH = BN * BK / 8 / 256;         // same for B when it is [N][K]
    constexpr int BT_UNITS = (BK / 8) * (BN / 4);    // 8x4 transpose units of a [K][N] tile
    constexpr int BT_U = (BT_UNITS + 255) / 256;     // ... per thread
    static_assert(A_CH >= 1 && (B_NK ? BN_CH >= 1 : BT_U >= 1), "tile too small for 256 threads");

    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* As = reinterpret_cast<bf16_t*>(smem);             // [2][BM][LD]
    bf16_t* Bs = As + 2 * BM * LD;                            // [2][BN][LD]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    A += (long)blockIdx.z * strideA;
    B += (long)blockIdx.z * strideB;
    const long c_off = (long)blockIdx.z * strideC;

    uint4 ra[A_CH];
    uint4 rbn[B_NK ? BN_CH : 1];
    uint2 rbt[B_NK ? 1 : BT_U][8];

    auto load_tile = [&](int k0) {
#pragma unroll
        for (int u = 0; u < A_CH; ++u) {
            const int c = tid + 256 * u, row = c / (BK / 8), kc = c % (BK / 8);
            const int gm = m0 + row, gk = k0 + kc * 8;
            ra[u] = (gm < M && gk < K) ? ld_u4(A + (long)gm * K + gk) : make_uint4(0, 0, 0, 0);
        }
        if constexpr (B_NK) {
#pragma unroll
            for (int u = 0; u < BN_CH; ++u) {
                const int c = tid + 256 * u, row = c / (BK / 8), kc = c % (BK / 8);
                const int gn = n0 + row, gk = k0 + kc * 8;
                rbn[u] = (gn < N && gk < K) ? ld_u4(B + (long)gn * K + gk) : make_uint4(0, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int u = 0; u < BT_U; ++u) {
                const int c = tid + 256 * u, nq = c % (BN / 4), ko = c / (BN / 4);
                const int gn = n0 + nq * 4;
                if (c >= BT_UNITS) continue;
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    const int gk = k0 + ko * 8 + kk;
                    rbt[u][kk] = (gn < N && gk < K)
                                     ? *reinterpret_cast<const uint2*>(B + (long)gk * N + gn)
                                     : make_uint2(0, 0);
                }
            }
        }
    };
    auto store_tile = [&](int buf) {
        bf16_t* as = As + buf * BM * LD;
        bf16_t* bs = Bs + buf * BN * LD;
#pragma unroll
        for (int u = 0; u < A_CH; ++u) {
            const int c = tid + 256 * u, row = c / (BK / 8), kc = c % (BK / 8);
            st_u4(as + row * LD + kc * 8, ra[u]);
        }
        if constexpr (B_NK) {
#pragma unroll
            for (int u = 0; u < BN_CH; ++u) {
                const int c = tid + 256 * u, row = c / (BK / 8), kc = c % (BK / 8);
                st_u4(bs + row * LD + kc * 8, rbn[u]);
            }
        } else {
#pragma unroll
            for (int u = 0; u < BT_U; ++u) {
                const int c = tid + 256 * u, nq = c % (BN / 4), ko = c / (BN / 4);
                if (c >= BT_UNITS) continue;
                uint4 t[4];
                transpose_8x4(rbt[u], t);
#pragma unroll
                for (int q = 0; q < 4; ++q) st_u4(bs + (nq * 4 + q) * LD + ko * 8, t[q]);
            }
        }
    };

    f32x16 acc[MT][NT];
    zero_acc(acc);

    const int nk = (K + BK - 1) / BK;
    load_tile(0);
    store_tile(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_tile((kt + 1) * BK);
        const bf16_t* as = As + buf * BM * LD + (wm * MT * 32) * LD;
        const bf16_t* bs = Bs + buf * BN * LD + (wn * NT * 32) * LD;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) wave_mma_k16<MT, NT>(acc, as + ks * 16, LD, bs + ks * 16, LD, lane);
        if (kt + 1 < nk) store_tile(buf ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds column j of each 32x32 tile, 16 rows
    const int j = lane & 31, h = lane >> 5;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int col = n0 + (wn * NT + n) * 32 + j;
        if (col >= N) continue;
        const float bv = bias ? bias[col] : 0.0f;
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + (wm * MT + m) * 32 + acc_row(r, h);
                if (row < M) {
                    float v = alpha * acc[m][n][r] + bv;
                    if (R) v += (float)R[c_off + (long)row * N + col];
                    v = apply_act_rt(v, act);
                    if constexpr (OUT_F32) reinterpret_cast<float*>(Cv)[c_off + (long)row * N + col] = v;
                    else reinterpret_cast<bf16_t*>(Cv)[c_off + (long)row * N + col] = (bf16_t)v;
                }
            }
    }
}

// ---------------------------------------------------------------------------------------
// fp32 GEMM on the fp32 matrix instruction (true fp32, no reduced-precision mode).
// Tile 64 x 64 per workgroup, 4 waves each 32 x 32 (v_mfma_f32_32x32x2_f32), K step 16.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gemm_f32_kernel(
    const float* __restrict__ A, const float* __restrict__ B, const float* __restrict__ bias,
    const float* __restrict__ R, float* __restrict__ C, int M, int K, int N, int act) {
    constexpr int BK = 16;
    __shared__ float As[64][BK + 1];
    __shared__ float Bs[BK][64 + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int i = lane & 31, h = lane >> 5;
    f32x16 acc = {0};
    for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = tid + 256 * u;
            const int ar = e / BK, ac = e % BK;
            As[ar][ac] = (m0 + ar < M && k0 + ac < K) ? A[(long)(m0 + ar) * K + k0 + ac] : 0.0f;
            const int br = e / 64, bc = e % 64;
            Bs[br][bc] = (k0 + br < K && n0 + bc < N) ? B[(long)(k0 + br) * N + n0 + bc] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(As[wm * 32 + i][kk + h], Bs[kk + h][wn * 32 + i], acc, 0, 0, 0);
        __syncthreads();
    }
    const int col = n0 + wn * 32 + i;
    if (col < N) {
        const float bv = bias ? bias[col] : 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = m0 + wm * 32 + acc_row(r, h);
            if (row < M) {
                float v = acc[r] + bv;
                if (R) v += R[(long)row * N + col];
                C[(long)row * N + col] = apply_act_rt(v, act);
            }
        }
    }
}

template <int BM, int BN, int WM, int WN, bool B_NK, bool OUT_F32 = false>
static hipError_t launch_gemm_bf16(const void* a, const void* b, const float* bias, const void* res, void* c, long batch,
                                   int M, int K, int N, int act, float alpha, hipStream_t s) {
    constexpr size_t smem = (size_t)2 * (BM + BN) * (64 + 8) * sizeof(bf16_t);
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, B_NK, OUT_F32>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM, (unsigned)batch);
    hipLaunchKernelGGL(kern, grid, dim3(256), smem, s, (const bf16_t*)a, (const bf16_t*)b, bias,
                       (const bf16_t*)res, c, M, K, N, act, alpha, (long)M * K, B_NK ? (long)N * K : (long)K * N,
                       (long)M * N);
    return hipGetLastError();
}

hipError_t gemm_bf16(const void* a, const void* b, const float* bias, const void* res, void* c, int M,
                     int K, int N, int act, hipStream_t s) {
    // Enough tiles to cover 256 CUs decides the tile: big tiles when the problem is big.
    const long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
    if (N <= 64) return launch_gemm_bf16<128, 64, 4, 1, false>(a, b, bias, res, c, 1, M, K, N, act, 1.0f, s);
    if (t128 >= 192) return launch_gemm_bf16<128, 128, 2, 2, false>(a, b, bias, res, c, 1, M, K, N, act, 1.0f, s);
    return launch_gemm_bf16<64, 128, 2, 2, false>(a, b, bias, res, c, 1, M, K, N, act, 1.0f, s);
}

hipError_t gemm_f32(const void* a, const void* b, const float* bias, const void* res, void* c, int M,
                    int K, int N, int act, hipStream_t s) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, s, (const float*)a, (const float*)b, bias,
                       (const float*)res, (float*)c, M, K, N, act);
    return hipGetLastError();
}

hipError_t bmm_nt_bf16(const void* a, const void* b, void* c, long batch, int M, int N, int K,
                       float alpha, bool out_f32, hipStream_t s) {
    if (out_f32) return launch_gemm_bf16<128, 128, 2, 2, true, true>(a, b, nullptr, nullptr, c, batch, M, K, N, kNone, alpha, s);
    return launch_gemm_bf16<128, 128, 2, 2, true>(a, b, nullptr, nullptr, c, batch, M, K, N, kNone, alpha, s);
}

hipError_t bmm_nn_bf16(const void* a, const void* b, void* c, long batch, int M, int N, int K,
                       hipStream_t s) {
    if (N <= 64) return launch_gemm_bf16<128, 64, 4, 1, false>(a, b, nullptr, nullptr, c, batch, M, K, N, kNone, 1.0f, s);
    return launch_gemm_bf16<64, 128, 2, 2, false>(a, b, nullptr, nullptr, c, batch, M, K, N, kNone, 1.0f, s);
}

}  // namespace ago
