// Fused matmul -> activation -> matmul (pw->pw, the "downstream pointwise" rule of AGO
// Sec. III-B / Fig. 7b: the downstream tile keeps all of its output channels, the upstream
// tile is a slice o1 of the hidden dimension, which is the downstream reduction dimension).
//
// Workgroup (s, rb) owns BM rows of X and the slice [s*FS, (s+1)*FS) of the hidden dimension:
//   phase 1  Hs[BM][FS] = act(X[rb] * W1[:, slice] + b1[slice])   -> bf16, stays in LDS
//   phase 2  P[s][rb]   = Hs * W2[slice, :]                        -> fp32 partial, all K2 columns
// The hidden activation never leaves the chip.  Because the slice is only part of the
// downstream reduction, the F/FS partial products are summed (deterministically, in slice
// order) by a second small kernel that also adds b2 and rounds to bf16.  With a single slice
// (F == FS) phase 2 writes y directly.
#include "ago_dev.hpp"
#include "ago_launch.hpp"

namespace ago {

// WF x WM1 = 4 waves in phase 1 (hidden x rows); WM2 x WN2 = 4 waves in phase 2 (rows x cols).
template <int BM, int FS, int WF, int WM1, int BN2, int WM2, int WN2>
struct FfnCfg {
    static constexpr int BK = 64, LD = BK + 8, LDH = FS + 8;
    static constexpr int FT = FS / WF / 32, MT1 = BM / WM1 / 32;   // phase-1 wave tile (f x m)
    static constexpr int MT2 = BM / WM2 / 32, NT2 = BN2 / WN2 / 32; // phase-2 wave tile (m x n)
    static constexpr int KT2 = FS / BK;
    static constexpr size_t kStage1 = (size_t)2 * (BM + FS) * LD * 2;
    static constexpr size_t kHs = (size_t)BM * LDH * 2;
    static constexpr size_t kStage2 = (size_t)2 * BN2 * LD * 2;
    static constexpr size_t kSmem = kStage1 > kHs + kStage2 ? kStage1 : kHs + kStage2;
    static_assert(WF * WM1 == 4 && WM2 * WN2 == 4, "4 waves");
    static_assert(FS % BK == 0 && FS % (WF * 32) == 0 && BM % (WM1 * 32) == 0, "phase-1 tiling");
    static_assert(BM % (WM2 * 32) == 0 && BN2 % (WN2 * 32) == 0, "phase-2 tiling");
    static_assert(kSmem <= 160 * 1024, "LDS");
};

template <class Cfg, int BM, int FS, int WF, int WM1, int BN2, int WM2, int WN2>
__global__ __launch_bounds__(256) void fused_ffn_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ W1, const float* __restrict__ b1,
    const bf16_t* __restrict__ W2, const float* __restrict__ b2, bf16_t* __restrict__ Y,
    float* __restrict__ part, int M, int K, int F, int K2, int act) {
    constexpr int BK = Cfg::BK, LD = Cfg::LD, LDH = Cfg::LDH;
    constexpr int FT = Cfg::FT, MT1 = Cfg::MT1, MT2 = Cfg::MT2, NT2 = Cfg::NT2, KT2 = Cfg::KT2;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* Xs = reinterpret_cast<bf16_t*>(smem);          // [2][BM][LD]   phase 1
    bf16_t* W1s = Xs + 2 * BM * LD;                        // [2][FS][LD]   phase 1
    bf16_t* Hs = reinterpret_cast<bf16_t*>(smem);          // [BM][LDH]     phase 2 (aliases phase-1 staging)
    bf16_t* W2s = Hs + BM * LDH;                           // [2][BN2][LD]  phase 2

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int split = blockIdx.x, nsplit = gridDim.x;
    const int m0 = blockIdx.y * BM, f0 = split * FS;

    // ------------------------------ phase 1 -------------------------------------------
    {
        constexpr int X_CH = BM * BK / 8 / 256;
        constexpr int W_UNITS = (BK / 8) * (FS / 4), W_U = (W_UNITS + 255) / 256;
        uint4 rx[X_CH];
        uint2 rw[W_U][8];
        auto load_tile = [&](int k0) {
#pragma unroll
            for (int u = 0; u < X_CH; ++u) {
                const int c = tid + 256 * u, row = c / (BK / 8), kc = c % (BK / 8);
                const int gm = m0 + row, gk = k0 + kc * 8;
                rx[u] = (gm < M && gk < K) ? ld_u4(X + (long)gm * K + gk) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < W_U; ++u) {
                const int c = tid + 256 * u, nq = c % (FS / 4), ko = c / (FS / 4);
                if (c >= W_UNITS) continue;
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    const int gk = k0 + ko * 8 + kk;
                    rw[u][kk] = gk < K ? *reinterpret_cast<const uint2*>(W1 + (long)gk * F + f0 + nq * 4)
                                       : make_uint2(0, 0);
                }
            }
        };
        auto store_tile = [&](int buf) {
#pragma unroll
            for (int u = 0; u < X_CH; ++u) {
                const int c = tid + 256 * u, row = c / (BK / 8), kc = c % (BK / 8);
                st_u4(Xs + (buf * BM + row) * LD + kc * 8, rx[u]);
            }
#pragma unroll
            for (int u = 0; u < W_U; ++u) {
                const int c = tid + 256 * u, nq = c % (FS / 4), ko = c / (FS / 4);
                if (c >= W_UNITS) continue;
                uint4 t[4];
                transpose_8x4(rw[u], t);
#pragma unroll
                for (int q = 0; q < 4; ++q) st_u4(W1s + (buf * FS + nq * 4 + q) * LD + ko * 8, t[q]);
            }
        };
        const int wf = wave / WM1, wm = wave % WM1;
        f32x16 acc[FT][MT1];   // rows = hidden units, cols = rows of X
        zero_acc(acc);
        const int nk = (K + BK - 1) / BK;
        load_tile(0);
        store_tile(0);
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            const int buf = kt & 1;
            if (kt + 1 < nk) load_tile((kt + 1) * BK);
            const bf16_t* as = W1s + (buf * FS + wf * FT * 32) * LD;
            const bf16_t* bs = Xs + (buf * BM + wm * MT1 * 32) * LD;
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks)
                wave_mma_k16<FT, MT1>(acc, as + ks * 16, LD, bs + ks * 16, LD, lane);
            if (kt + 1 < nk) store_tile(buf ^ 1);
            __syncthreads();
        }
        // epilogue: bias + activation, round to bf16, Hs[m][f] (f contiguous = phase-2 k)
        const int j = lane & 31, h = lane >> 5;
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int fl = (wf * FT + ft) * 32 + 8 * g + 4 * h;   // local hidden index of 4 regs
                float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
                if (b1) bv = *reinterpret_cast<const float4*>(b1 + f0 + fl);
#pragma unroll
                for (int mt = 0; mt < MT1; ++mt) {
                    const int ml = (wm * MT1 + mt) * 32 + j;
                    const float v0 = apply_act_rt(acc[ft][mt][4 * g + 0] + bv.x, act);
                    const float v1 = apply_act_rt(acc[ft][mt][4 * g + 1] + bv.y, act);
                    const float v2 = apply_act_rt(acc[ft][mt][4 * g + 2] + bv.z, act);
                    const float v3 = apply_act_rt(acc[ft][mt][4 * g + 3] + bv.w, act);
                    *reinterpret_cast<uint2*>(Hs + ml * LDH + fl) = make_uint2(pack_bf16(v0, v1), pack_bf16(v2, v3));
                }
            }
    }

    // ------------------------------ phase 2 -------------------------------------------
    {
        constexpr int W_UNITS = (BK / 8) * (BN2 / 4), W_U = (W_UNITS + 255) / 256;
        uint2 rw[W_U][8];
        const int NB = K2 / BN2, T = NB * KT2;
        auto load_tile = [&](int t) {
            const int nb = t / KT2, kt = t % KT2;
#pragma unroll
            for (int u = 0; u < W_U; ++u) {
                const int c = tid + 256 * u, nq = c % (BN2 / 4), ko = c / (BN2 / 4);
                if (c >= W_UNITS) continue;
#pragma unroll
                for (int kk = 0; kk < 8; ++kk)
                    rw[u][kk] = *reinterpret_cast<const uint2*>(
                        W2 + (long)(f0 + kt * BK + ko * 8 + kk) * K2 + nb * BN2 + nq * 4);
            }
        };
        auto store_tile = [&](int buf) {
#pragma unroll
            for (int u = 0; u < W_U; ++u) {
                const int c = tid + 256 * u, nq = c % (BN2 / 4), ko = c / (BN2 / 4);
                if (c >= W_UNITS) continue;
                uint4 t4[4];
                transpose_8x4(rw[u], t4);
#pragma unroll
                for (int q = 0; q < 4; ++q) st_u4(W2s + (buf * BN2 + nq * 4 + q) * LD + ko * 8, t4[q]);
            }
        };
        const int wm = wave / WN2, wn = wave % WN2;
        const int j = lane & 31, h = lane >> 5;
        f32x16 acc[MT2][NT2];  // rows = rows of X, cols = output columns
        zero_acc(acc);
        load_tile(0);
        store_tile(0);
        __syncthreads();       // also publishes Hs
        for (int t = 0; t < T; ++t) {
            const int buf = t & 1, nb = t / KT2, kt = t % KT2;
            if (t + 1 < T) load_tile(t + 1);
            const bf16_t* as = Hs + (wm * MT2 * 32) * LDH + kt * BK;
            const bf16_t* bs = W2s + (buf * BN2 + wn * NT2 * 32) * LD;
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks)
                wave_mma_k16<MT2, NT2>(acc, as + ks * 16, LDH, bs + ks * 16, LD, lane);
            if (kt == KT2 - 1) {
#pragma unroll
                for (int nt = 0; nt < NT2; ++nt) {
                    const int col = nb * BN2 + (wn * NT2 + nt) * 32 + j;
#pragma unroll
                    for (int mt = 0; mt < MT2; ++mt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int row = m0 + (wm * MT2 + mt) * 32 + acc_row(r, h);
                            if (row < M) {
                                if (nsplit == 1) Y[(long)row * K2 + col] = (bf16_t)(acc[mt][nt][r] + (b2 ? b2[col] : 0.0f));
                                else part[((long)split * M + row) * K2 + col] = acc[mt][nt][r];
                            }
                            acc[mt][nt][r] = 0.0f;
                        }
                }
            }
            if (t + 1 < T) store_tile(buf ^ 1);
            __syncthreads();
        }
    }
}

// y[m][n] = bf16( sum_s part[s][m][n] + b2[n] ), slices added in index order.
__global__ __launch_bounds__(256) void ffn_reduce_kernel(const float* __restrict__ part,
                                                         const float* __restrict__ b2,
                                                         bf16_t* __restrict__ Y, long MK2, int K2, int nsplit) {
    const long n4 = MK2 / 4;
    for (long i = blockIdx.x * 256L + threadIdx.x; i < n4; i += (long)gridDim.x * 256) {
        float4 a = reinterpret_cast<const float4*>(part)[i];
        for (int s = 1; s < nsplit; ++s) {
            const float4 v = reinterpret_cast<const float4*>(part + (long)s * MK2)[i];
            a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
        }
        if (b2) {
            const float4 bv = *reinterpret_cast<const float4*>(b2 + (int)((i * 4) % K2));
            a.x += bv.x; a.y += bv.y; a.z += bv.z; a.w += bv.w;
        }
        reinterpret_cast<uint2*>(Y)[i] = make_uint2(pack_bf16(a.x, a.y), pack_bf16(a.z, a.w));
    }
}

template <int BM, int FS, int WF, int WM1, int BN2, int WM2, int WN2>
static hipError_t launch_ffn(const void* x, const void* w1, const float* b1, const void* w2,
                             const float* b2, void* y, int M, int K, int F, int K2, int act,
                             void* workspace, hipStream_t s) {
    typedef FfnCfg<BM, FS, WF, WM1, BN2, WM2, WN2> Cfg;
    auto kern = fused_ffn_kernel<Cfg, BM, FS, WF, WM1, BN2, WM2, WN2>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)Cfg::kSmem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int nsplit = F / FS;
    dim3 grid(nsplit, (M + BM - 1) / BM);
    prof_start(2, s);
    hipLaunchKernelGGL(kern, grid, dim3(256), Cfg::kSmem, s, (const bf16_t*)x, (const bf16_t*)w1, b1,
                       (const bf16_t*)w2, b2, (bf16_t*)y, (float*)workspace, M, K, F, K2, act);
    prof_stop(2, s);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || nsplit == 1) return e;
    const long MK2 = (long)M * K2;
    long g = (MK2 / 4 + 255) / 256;
    if (g > 2048) g = 2048;
    hipLaunchKernelGGL(ffn_reduce_kernel, dim3((unsigned)g), dim3(256), 0, s, (const float*)workspace, b2,
                       (bf16_t*)y, MK2, K2, nsplit);
    return hipGetLastError();
}

// Tile configurations (BM rows, FS hidden slice, phase-2 column block):
//   0: 128 x 192, 128   1: 64 x 384, 256   2: 128 x 128, 128   3: 128 x 64, 64 (small shapes)
int fused_ffn_num_cfgs() { return 4; }

static bool ffn_cfg_ok(int cfg, int F, int K2) {
    switch (cfg) {
        case 0: return F % 192 == 0 && K2 % 128 == 0;
        case 1: return F % 384 == 0 && K2 % 256 == 0;
        case 2: return F % 128 == 0 && K2 % 128 == 0;
        case 3: return F % 64 == 0 && K2 % 64 == 0;
        default: return false;
    }
}

int fused_ffn_pick_cfg(int M, int K, int F, int K2, int tile_cfg) {
    (void)M; (void)K;
    if (tile_cfg >= 0) return ffn_cfg_ok(tile_cfg, F, K2) ? tile_cfg : -1;
    for (int c = 0; c < 4; ++c)
        if (ffn_cfg_ok(c, F, K2)) return c;
    return -1;
}

int fused_ffn_nsplit(int cfg, int F) {
    static const int fs[4] = {192, 384, 128, 64};
    return (cfg >= 0 && cfg < 4) ? F / fs[cfg] : 0;
}

hipError_t fused_ffn(const void* x, const void* w1, const float* b1, const void* w2, const float* b2,
                     void* y, int M, int K, int F, int K2, int act, int tile_cfg, void* workspace,
                     hipStream_t s) {
    switch (fused_ffn_pick_cfg(M, K, F, K2, tile_cfg)) {
        case 0: return launch_ffn<128, 192, 2, 2, 128, 2, 2>(x, w1, b1, w2, b2, y, M, K, F, K2, act, workspace, s);
        case 1: return launch_ffn<64, 384, 4, 1, 256, 1, 4>(x, w1, b1, w2, b2, y, M, K, F, K2, act, workspace, s);
        case 2: return launch_ffn<128, 128, 2, 2, 128, 2, 2>(x, w1, b1, w2, b2, y, M, K, F, K2, act, workspace, s);
        case 3: return launch_ffn<128, 64, 1, 4, 64, 4, 1>(x, w1, b1, w2, b2, y, M, K, F, K2, act, workspace, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ago
