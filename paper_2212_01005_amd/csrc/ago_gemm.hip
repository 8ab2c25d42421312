// Un-fused matrix products (one complex operator per kernel, optional epilogue):
// ago_gemm / ago_conv1x1 (bf16 and fp32), ago_bmm_nt, ago_bmm_nn.
#include "ago_dev.hpp"
#include "ago_launch.hpp"
#include "ago_mma_tile.hpp"

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
    long strideA, long strideB, long strideC, int lda, int ldc) {
    // lda / ldc: elements per row of A / C (>= K / N; a padded row's tail must hold zeros in A)
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
            ra[u] = (gm < M && gk < K) ? ld_u4(A + (long)gm * lda + gk) : make_uint4(0, 0, 0, 0);
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
                    if (R) v += (float)R[c_off + (long)row * ldc + col];
                    v = apply_act_rt(v, act);
                    if constexpr (OUT_F32) reinterpret_cast<float*>(Cv)[c_off + (long)row * ldc + col] = v;
                    else reinterpret_cast<bf16_t*>(Cv)[c_off + (long)row * ldc + col] = (bf16_t)v;
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


// ---------------------------------------------------------------------------------------
// bf16 GEMM for shapes that tile exactly: C[M][N] = act(A[M][K] * B[K][N] + bias) (+ R).
// Eight waves, each with a 64 x 96 accumulator tile; KS of them share one output tile and split every
// BK-deep LDS tile along k (wave kh takes k16 steps kh * KPW .. + KPW - 1), so a 128 x 192 (KS = 2)
// or 64 x 96 (KS = 8) workgroup tile still gives every wave the 64 x 96 shape whose weight fragments
// (transposing LDS reads) feed two matrix instructions each.  The k-partials meet in LDS at the end,
// summed in wave order.  Both operands travel global -> registers -> LDS in their natural layouts, two
// tiles in flight in registers ahead of the one being multiplied (LDS is double-buffered).
// Launch index -> tile: each XCD (launch index mod 8) takes panels of 8 row tiles x TN / ... column
// tiles so that the A rows and B columns it touches stay in its L2.
// ---------------------------------------------------------------------------------------
template <int BM_, int BN_, int KS_, int KPW_>
struct KsplitCfg {
    static constexpr int BM = BM_, BN = BN_, KS = KS_, KPW = KPW_;
    static constexpr int WMG = BM / 64, WNG = BN / 96;
    static_assert(WMG * WNG * KS == 8 && BM % 64 == 0 && BN % 96 == 0, "eight waves of 64 x 96");
    static constexpr int BK = 16 * KPW * KS;
    static constexpr int A_STRIDE = BK * 2 + 16;
    static constexpr int W_STRIDE = BN * 2 + ((64 - (BN * 2) % 256) + 256) % 256;     // = 64 mod 256
    static constexpr int A_BYTES = BM * A_STRIDE, W_BYTES = BK * W_STRIDE, STAGE = A_BYTES + W_BYTES;
    static constexpr int A_CH = BM * BK / 8 / 512, W_CH = BK * BN / 8 / 512;        // 16-byte chunks per thread and tile
    static_assert(A_CH * 512 * 8 == BM * BK && W_CH * 512 * 8 == BK * BN, "tiles split evenly over 512 threads");
    static constexpr int RED_LD = 104;                                              // floats per row of a parked 32 x 96 tile
    static constexpr int RED_BYTES = 8 * 32 * RED_LD * 4;
    static constexpr int SMEM = 2 * STAGE > RED_BYTES ? 2 * STAGE : RED_BYTES;
    static_assert(W_STRIDE % 256 == 64 && SMEM <= 160 * 1024, "LDS layout");
};

template <int BM, int BN, int KS, int KPW>
__global__ __launch_bounds__(512) void gemm_bf16_ksplit_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, const float* __restrict__ bias,
    const bf16_t* __restrict__ R, bf16_t* __restrict__ C, int M, int K, int N, int act) {
    typedef KsplitCfg<BM, BN, KS, KPW> G;
    extern __shared__ __align__(16) unsigned char smem[];
    lds_u8* lds = (lds_u8*)smem;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kh = wave % KS, grp = wave / KS, wn = grp % G::WNG, wm = grp / G::WNG;

    // launch index -> (row tile, column tile)
    const int TM = M / BM, TN = N / BN, T = TM * TN;
    int j = blockIdx.x;
    if (T % 8 == 0) j = (blockIdx.x & 7) * (T / 8) + (blockIdx.x >> 3);     // an XCD takes T / 8 consecutive tiles
    int tm, tn;
    if (TM % 8 == 0) { tm = (j & 7) + 8 * (j / (8 * TN)); tn = (j >> 3) % TN; }   // panels of 8 row tiles, column tiles inside
    else { tm = j / TN; tn = j % TN; }
    const int m0 = tm * BM, n0 = tn * BN;

    // Chunk (16 bytes) ownership: A chunk u of a thread is 512 / (BK / 8) rows below chunk u - 1; the W
    // chunks of a thread lie in one k-row, CPR chunks apart.  All later addresses are a per-thread base
    // plus compile-time constants.
    constexpr int A_CPR = G::BK / 8, A_ROWS = 512 / A_CPR, CPR = (BN / 8) / G::W_CH;
    static_assert(512 / CPR == G::BK && 512 % A_CPR == 0, "chunk ownership");
    const int arow = tid / A_CPR, akc = tid % A_CPR, wk = tid / CPR, wnc = tid % CPR;
    const bf16_t* pa = A + (long)(m0 + arow) * K + akc * 8;
    const bf16_t* pw = B + (long)wk * N + n0 + wnc * 8;
    const long a_step = (long)A_ROWS * K;
    const int sa = arow * G::A_STRIDE + akc * 16;
    const int sw = G::A_BYTES + wk * G::W_STRIDE + wnc * 16;
    struct Regs { u32x4_t a[G::A_CH], w[G::W_CH]; };
    auto gload = [&](Regs& r, int kt) {
        const bf16_t* qa = pa + kt * G::BK;
        const bf16_t* qw = pw + (long)kt * G::BK * N;
#pragma unroll
        for (int u = 0; u < G::A_CH; ++u) r.a[u] = ldg16(qa + u * a_step);
#pragma unroll
        for (int u = 0; u < G::W_CH; ++u) r.w[u] = ldg16(qw + u * CPR * 8);
    };
    auto lstore = [&](const Regs& r, int stage) {
        lds_u8* st = lds + stage * G::STAGE;
#pragma unroll
        for (int u = 0; u < G::A_CH; ++u) lds_write16(st + sa + u * A_ROWS * G::A_STRIDE, r.a[u]);
#pragma unroll
        for (int u = 0; u < G::W_CH; ++u) lds_write16(st + sw + u * CPR * 16, r.w[u]);
    };
    const int aoff = a_frag_off(lane, wm * 64, kh * KPW * 16, G::A_STRIDE);
    const int woff = G::A_BYTES + w_frag_off(lane, wn * 96, kh * KPW * 16, G::W_STRIDE);
    f32x16 acc[2][3];
    zero_acc(acc);
    auto fetch = [&](Frag64x96& f, int stage, int ks) {
        const lds_u8* st = lds + stage * G::STAGE;
#pragma unroll
        for (int m = 0; m < 2; ++m) f.a[m] = lds_read_a(st + aoff + m * 32 * G::A_STRIDE + ks * 32);
#pragma unroll
        for (int n = 0; n < 3; ++n) f.w[n] = lds_read_w(st + woff + n * 64 + ks * 16 * G::W_STRIDE, G::W_STRIDE);
    };
    // One pass over the tile in LDS stage `stage`: fetch its fragments, request the tile three ahead, park the
    // next tile (in registers since two passes ago) in the other stage, multiply.  The order is pinned: the
    // loads go out first, the LDS stores issue between the matrix instructions of the two k steps.
    auto pass = [&](int stage, Regs& r, int kt_next) {
        Frag64x96 f0, f1;
        fetch(f0, stage, 0);
        if constexpr (KPW == 2) fetch(f1, stage, 1);
        __builtin_amdgcn_sched_barrier(0);
        lstore(r, stage ^ 1);
        __builtin_amdgcn_sched_barrier(0);
        gload(r, kt_next);
        __builtin_amdgcn_sched_barrier(0);
        mma_64x96(acc, f0);
        if constexpr (KPW == 2) mma_64x96(acc, f1);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    };

    const int nk = K / G::BK;
    Regs r0, r1;
    gload(r0, 0);
    lstore(r0, 0);
    gload(r1, min(1, nk - 1));
    gload(r0, min(2, nk - 1));
    __syncthreads();
    // loads past the end repeat the last tile (never used)
    int t = 0;
    for (; t + 1 < nk; t += 2) {
        pass(0, r1, min(t + 3, nk - 1));
        pass(1, r0, min(t + 4, nk - 1));
    }
    if (t < nk) pass(0, r1, nk - 1);

    // k-partials -> LDS, one 32-row tile of every wave at a time; the KS waves of an output tile then
    // each finish 32 / KS rows: partials added in wave order, bias, residual, activation, 8-byte stores
    float* red = reinterpret_cast<float*>(smem);
    const int jcol = lane & 31, h = lane >> 5;
    constexpr int RS = 32 / KS;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        float* mine = red + wave * 32 * G::RED_LD;
#pragma unroll
        for (int n = 0; n < 3; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) mine[acc_row(r, h) * G::RED_LD + n * 32 + jcol] = acc[mt][n][r];
        __syncthreads();
        for (int u = lane; u < RS * 24; u += 64) {
            const int row = kh * RS + u / 24, c4 = (u % 24) * 4;
            const float* src = red + (grp * KS) * 32 * G::RED_LD + row * G::RED_LD + c4;
            float4 v = *reinterpret_cast<const float4*>(src);
#pragma unroll
            for (int q = 1; q < KS; ++q) {
                const float4 w = *reinterpret_cast<const float4*>(src + q * 32 * G::RED_LD);
                v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
            }
            const int grow = m0 + wm * 64 + mt * 32 + row, gcol = n0 + wn * 96 + c4;
            if (bias) {
                const float4 bv = *reinterpret_cast<const float4*>(bias + gcol);
                v.x += bv.x; v.y += bv.y; v.z += bv.z; v.w += bv.w;
            }
            if (R) {
                const uint2 rv = *reinterpret_cast<const uint2*>(R + (long)grow * N + gcol);
                v.x += lo_bf16(rv.x); v.y += hi_bf16(rv.x); v.z += lo_bf16(rv.y); v.w += hi_bf16(rv.y);
            }
            v.x = apply_act_rt(v.x, act); v.y = apply_act_rt(v.y, act);
            v.z = apply_act_rt(v.z, act); v.w = apply_act_rt(v.w, act);
            *reinterpret_cast<uint2*>(C + (long)grow * N + gcol) = make_uint2(pack_bf16(v.x, v.y), pack_bf16(v.z, v.w));
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------
// Small products (a 1 x 1 convolution of one image, a projection with few rows): too little work for
// the LDS-tiled kernels above, whose few workgroups would each walk the whole reduction serially.
// Here an output tile is 32 x 32 and KS of the workgroup's eight waves split its reduction, so that even
// a 196 x 32 output keeps 56 waves busy; operands go global -> registers directly (they are read once
// per tile row / column and the whole problem sits in the caches), products run on the fp32 matrix
// instruction (bf16 inputs are widened first, exactly), partial sums meet in LDS in wave order.
// Lane (i, h) of v_mfma_f32_32x32x2_f32 supplies row / column i at reduction index h: the wave gives
// h = 0 the first half of its k range and h = 1 the second, so every lane walks consecutive k.
// ---------------------------------------------------------------------------------------
template <typename T> __device__ __forceinline__ float widen(T v) { return (float)v; }

template <typename T, int KS>
__global__ __launch_bounds__(512) void gemm_small_kernel(
    const T* __restrict__ A, const T* __restrict__ B, const float* __restrict__ bias,
    const T* __restrict__ R, T* __restrict__ C, int M, int K, int N, int act) {
    constexpr int TPW = 8 / KS, LD = 33;
    __shared__ float red[8][32 * LD];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kh = wave % KS, grp = wave / KS;
    const int tiles_n = (N + 31) / 32, tiles_m = (M + 31) / 32;
    const int tile = blockIdx.x * TPW + grp;
    const bool live = tile < tiles_m * tiles_n;                 // uniform per wave
    const int m0 = (tile / tiles_n) * 32, n0 = (tile % tiles_n) * 32;
    const int i = lane & 31, h = lane >> 5;

    f32x16 acc = {0};
    if (live) {
        const int per = (K + 2 * KS - 1) / (2 * KS);            // reduction indices per lane
        const int k_lo = (2 * kh + h) * per;
        const int row = m0 + i, col = n0 + i;
        const bool row_ok = row < M, col_ok = col < N;
        const T* pa = A + (long)(row_ok ? row : 0) * K;
        const T* pb = B + (col_ok ? col : 0);
        for (int s0 = 0; s0 < per; s0 += 8) {
            float av[8], bv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int k = k_lo + s0 + u;
                const bool ok = s0 + u < per && k < K;
                const int kc = ok ? k : 0;
                const float a = widen(pa[kc]), b = widen(pb[(long)kc * N]);
                av[u] = ok && row_ok ? a : 0.0f;
                bv[u] = ok && col_ok ? b : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u], bv[u], acc, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) red[wave][acc_row(r, h) * LD + i] = acc[r];
    }
    __syncthreads();
    if (!live) return;
    // the KS waves of a tile each finish 32 / KS of its rows
    constexpr int RS = 32 / KS;
    for (int u = lane; u < RS * 32; u += 64) {
        const int rr = kh * RS + u / 32, cc = u % 32;
        const int row = m0 + rr, col = n0 + cc;
        if (row >= M || col >= N) continue;
        float v = red[grp * KS][rr * LD + cc];
#pragma unroll
        for (int q = 1; q < KS; ++q) v += red[grp * KS + q][rr * LD + cc];
        if (bias) v += bias[col];
        if (R) v += widen(R[(long)row * N + col]);
        C[(long)row * N + col] = (T)apply_act_rt(v, act);
    }
}

template <typename T>
static hipError_t launch_gemm_small(const void* a, const void* b, const float* bias, const void* res, void* c,
                                    int M, int K, int N, int act, hipStream_t s) {
    const int tiles = ((M + 31) / 32) * ((N + 31) / 32);
#define AGO_SMALL(KS)                                                                                         \
    hipLaunchKernelGGL((gemm_small_kernel<T, KS>), dim3((tiles * KS + 7) / 8), dim3(512), 0, s, (const T*)a,   \
                       (const T*)b, bias, (const T*)res, (T*)c, M, K, N, act)
    if (K >= 64) AGO_SMALL(8);
    else if (K >= 32) AGO_SMALL(4);
    else if (K >= 16) AGO_SMALL(2);
    else AGO_SMALL(1);
#undef AGO_SMALL
    return hipGetLastError();
}

// A product this small is bound by latency, not by the matrix cores: it takes the direct kernel.
static bool is_small_product(int M, int K, int N) { return (long)M * K * N <= (1L << 25); }

template <int BM, int BN, int KS, int KPW>
static hipError_t launch_gemm_ksplit(const void* a, const void* b, const float* bias, const void* res, void* c,
                                     int M, int K, int N, int act, hipStream_t s) {
    typedef KsplitCfg<BM, BN, KS, KPW> G;
    auto kern = gemm_bf16_ksplit_kernel<BM, BN, KS, KPW>;
    if (hipError_t e = allow_dynamic_lds<gemm_bf16_ksplit_kernel<BM, BN, KS, KPW>>(G::SMEM); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((M / BM) * (N / BN)), dim3(512), G::SMEM, s, (const bf16_t*)a, (const bf16_t*)b, bias,
                       (const bf16_t*)res, (bf16_t*)c, M, K, N, act);
    return hipGetLastError();
}

template <int BM, int BN, int WM, int WN, bool B_NK, bool OUT_F32 = false>
static hipError_t launch_gemm_bf16(const void* a, const void* b, const float* bias, const void* res, void* c, long batch,
                                   int M, int K, int N, int act, float alpha, hipStream_t s, int lda = 0, int ldc = 0) {
    if (lda == 0) lda = K;
    if (ldc == 0) ldc = N;
    constexpr size_t smem = (size_t)2 * (BM + BN) * (64 + 8) * sizeof(bf16_t);
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, B_NK, OUT_F32>;
    if (hipError_t e = allow_dynamic_lds<gemm_bf16_kernel<BM, BN, WM, WN, B_NK, OUT_F32>>((int)((int)smem)); e != hipSuccess) return e;
    dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM, (unsigned)batch);
    hipLaunchKernelGGL(kern, grid, dim3(256), smem, s, (const bf16_t*)a, (const bf16_t*)b, bias,
                       (const bf16_t*)res, c, M, K, N, act, alpha, (long)M * lda, B_NK ? (long)N * K : (long)K * N,
                       (long)M * ldc, lda, ldc);
    return hipGetLastError();
}

hipError_t gemm_bf16(const void* a, const void* b, const float* bias, const void* res, void* c, int M,
                     int K, int N, int act, hipStream_t s) {
    if (is_small_product(M, K, N)) return launch_gemm_small<bf16_t>(a, b, bias, res, c, M, K, N, act, s);
    // Shapes that tile exactly take the k-split kernels: 128 x 192 tiles when they fill the chip, else
    // 64 x 96 tiles whose eight waves split k (a product with few outputs and a long reduction).
    if (M % 128 == 0 && N % 192 == 0 && K % 64 == 0 && (long)(M / 128) * (N / 192) >= 192)
        return launch_gemm_ksplit<128, 192, 2, 2>(a, b, bias, res, c, M, K, N, act, s);
    if (M % 64 == 0 && N % 96 == 0 && K % 128 == 0 && (long)(M / 64) * (N / 96) >= 128)
        return launch_gemm_ksplit<64, 96, 8, 1>(a, b, bias, res, c, M, K, N, act, s);
    // Enough tiles to cover 256 CUs decides the tile: big tiles when the problem is big.
    const long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
    if (N <= 64) return launch_gemm_bf16<128, 64, 4, 1, false>(a, b, bias, res, c, 1, M, K, N, act, 1.0f, s);
    if (t128 >= 192) return launch_gemm_bf16<128, 128, 2, 2, false>(a, b, bias, res, c, 1, M, K, N, act, 1.0f, s);
    return launch_gemm_bf16<64, 128, 2, 2, false>(a, b, bias, res, c, 1, M, K, N, act, 1.0f, s);
}

hipError_t gemm_f32(const void* a, const void* b, const float* bias, const void* res, void* c, int M,
                    int K, int N, int act, hipStream_t s) {
    if (is_small_product(M, K, N)) return launch_gemm_small<float>(a, b, bias, res, c, M, K, N, act, s);
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, s, (const float*)a, (const float*)b, bias,
                       (const float*)res, (float*)c, M, K, N, act);
    return hipGetLastError();
}

hipError_t bmm_nt_bf16(const void* a, const void* b, void* c, long batch, int M, int N, int K,
                       float alpha, bool out_f32, hipStream_t s, int ldc) {
    if (out_f32) return launch_gemm_bf16<128, 128, 2, 2, true, true>(a, b, nullptr, nullptr, c, batch, M, K, N, kNone, alpha, s, 0, ldc);
    return launch_gemm_bf16<128, 128, 2, 2, true>(a, b, nullptr, nullptr, c, batch, M, K, N, kNone, alpha, s, 0, ldc);
}

hipError_t bmm_nn_bf16(const void* a, const void* b, void* c, long batch, int M, int N, int K,
                       hipStream_t s, int lda) {
    if (N <= 64) return launch_gemm_bf16<128, 64, 4, 1, false>(a, b, nullptr, nullptr, c, batch, M, K, N, kNone, 1.0f, s, lda);
    return launch_gemm_bf16<64, 128, 2, 2, false>(a, b, nullptr, nullptr, c, batch, M, K, N, kNone, 1.0f, s, lda);
}

}  // namespace ago
