// Fused matmul -> activation -> matmul (pw->pw, the "downstream pointwise" rule of AGO
// Sec. III-B / Fig. 7b: the downstream tile keeps all of its output channels, the upstream
// tile is a slice o1 of the hidden dimension, which is the downstream reduction dimension).
//
// Workgroup (s, rb), 8 waves, owns BM rows of X and the slice [s*FS, (s+1)*FS) of the hidden
// dimension:
//   phase 1  Hs[BM][FS] = act(X[rb] * W1[:, slice] + b1[slice])   -> bf16, stays in LDS
//   phase 2  P[s][rb]   = Hs * W2[slice, :]                        -> fp32 partial, all K2 columns
// The hidden activation never leaves the chip.  Because the slice is only part of the
// downstream reduction, the F/FS partial products are summed (deterministically, in slice
// order) by a second small kernel that also adds b2 and rounds to bf16.  With a single slice
// (F == FS) phase 2 writes y directly.
//
// Both phases run the same software pipeline over 64-deep k-tiles:
//   global -> registers two tiles ahead, registers -> LDS one tile ahead (weights transposed to
//   [n][k] and chunk-swizzled on the way), LDS -> MFMA fragments one k16 step ahead, one
//   barrier per tile.  Two register sets and two LDS buffers alternate (loop unrolled by two).
#include "ago_dev.hpp"
#include "ago_launch.hpp"

namespace ago {

constexpr int kFfnThreads = 512;

// Stage a [KD k][BN n] tile of a row-major [K][N] matrix into LDS as [n][k] (k contiguous, KD + 8
// elements per row, 16-byte chunk index XOR-ed with (n >> 4) & 3): 8x4 transposition units,
// unit u -> n-quad u % (BN/4), k-octet u / (BN/4).
template <int BN, int KD = 64>
struct WeightStager {
    static constexpr int UNITS = (KD / 8) * (BN / 4), LDW = KD + 8;
    static constexpr int U = (UNITS + kFfnThreads - 1) / kFfnThreads;
    uint2 r[U][8];
    // No bounds checks and no predication: the caller guarantees that the whole [64][BN] tile lies
    // inside W, and every thread issues the same number of loads.  (A conditional load inside the
    // pipelined loop would make the compiler wait for *all* outstanding loads at the next use.)
    __device__ __forceinline__ void load(const bf16_t* W, long ldw, int k0, int n0, int tid) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = (tid + kFfnThreads * u) % UNITS;   // surplus threads repeat a unit (never stored)
            const int nq = c % (BN / 4), ko = c / (BN / 4);
            const bf16_t* src = W + (long)(k0 + ko * 8) * ldw + n0 + nq * 4;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) r[u][kk] = *reinterpret_cast<const uint2*>(src + kk * ldw);
        }
    }
    __device__ __forceinline__ void store_unit(bf16_t* dst, int tid, int u) const {
        const int c = tid + kFfnThreads * u;
        if (UNITS % kFfnThreads != 0 && c >= UNITS) return;
        const int nq = c % (BN / 4), ko = c / (BN / 4);
        uint4 t[4];
        transpose_8x4(r[u], t);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = nq * 4 + q;
            st_u4(dst + n * LDW + ((ko ^ ((n >> 4) & 3)) << 3), t[q]);
        }
    }
    __device__ __forceinline__ void store(bf16_t* dst, int tid) const {
#pragma unroll
        for (int u = 0; u < U; ++u) store_unit(dst, tid, u);
    }
};

// Stage a [BM m][64 k] tile of a row-major [M][K] matrix into LDS as [m][k], 72 elements per row.
template <int BM>
struct ActStager {
    static constexpr int CH = BM * 8 / kFfnThreads;
    static_assert(CH >= 1, "tile too small");
    uint4 r[CH];
    // Rows beyond M are clamped to the last row (their results are never stored); k0 + 64 <= K.
    __device__ __forceinline__ void load(const bf16_t* X, int K, int m0, int k0, int M, int tid) {
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int c = tid + kFfnThreads * u, row = c >> 3, kc = c & 7;
            const int gm = min(m0 + row, M - 1);
            r[u] = ld_u4(X + (long)gm * K + k0 + kc * 8);
        }
    }
    __device__ __forceinline__ void store(bf16_t* dst, int tid) const {
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int c = tid + kFfnThreads * u, row = c >> 3, kc = c & 7;
            st_u4(dst + row * 72 + kc * 8, r[u]);
        }
    }
};

// Fragments of one k16 step of a wave tile: NW row tiles of a swizzled weight tile (row stride ldw
// elements) and NA row tiles of a plain activation tile (row stride lda elements).
template <int NW, int NA>
struct Frags {
    bf16x8 w[NW], a[NA];
    // ws points at the weight tile's row 0; w0 = first row of this wave (a multiple of 32)
    __device__ __forceinline__ void fetch(const bf16_t* ws, int ldw, int w0, const bf16_t* as, int lda, int ks, int i, int h) {
#pragma unroll
        for (int t = 0; t < NW; ++t) {
            const int row = w0 + t * 32 + i;
            w[t] = ld_bf16x8(ws + row * ldw + (((ks * 2 + h) ^ ((row >> 4) & 3)) << 3));
        }
#pragma unroll
        for (int t = 0; t < NA; ++t) a[t] = ld_bf16x8(as + (t * 32 + i) * lda + ks * 16 + 8 * h);
    }
};

template <int BM, int FS, int BN2>
struct FfnCfg {
    static constexpr int BK = 64, LD = 72, LDH = FS + 8;
    // phase 1: 2 (hidden) x 4 (rows) waves; phase 2: 2 (rows) x 4 (cols) waves
    static constexpr int FT = FS / 2 / 32, MT1 = BM / 4 / 32;
    static constexpr int MT2 = BM / 2 / 32, NT2 = BN2 / 4 / 32;
    static constexpr size_t kStage1 = (size_t)2 * (BM + FS) * LD * 2;
    static constexpr size_t kHs = (size_t)BM * LDH * 2;
    static constexpr size_t kStage2 = (size_t)2 * BN2 * LDH * 2;   // phase-2 tiles span the whole slice
    static constexpr size_t kMain = kStage1 > kHs + kStage2 ? kStage1 : kHs + kStage2;
    static constexpr size_t kSmem = kMain + FS * 4;      // + b1 slice
    static_assert(FS % 64 == 0 && BM % 128 == 0 && BN2 % 128 == 0, "tiling");
    static_assert((FS / 2) % 32 == 0, "each phase-1 wave row must start on a multiple of 32 hidden units");
    static_assert(kSmem <= 160 * 1024, "LDS");
};

template <int BM, int FS, int BN2>
__global__ __launch_bounds__(kFfnThreads) void fused_ffn_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ W1, const float* __restrict__ b1,
    const bf16_t* __restrict__ W2, const float* __restrict__ b2, bf16_t* __restrict__ Y,
    float* __restrict__ part, int M, int K, int F, int K2, int act) {
    typedef FfnCfg<BM, FS, BN2> Cfg;
    constexpr int BK = Cfg::BK, LD = Cfg::LD, LDH = Cfg::LDH;
    constexpr int FT = Cfg::FT, MT1 = Cfg::MT1, MT2 = Cfg::MT2, NT2 = Cfg::NT2;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* Xs = reinterpret_cast<bf16_t*>(smem);          // [2][BM][LD]   phase 1
    bf16_t* W1s = Xs + 2 * BM * LD;                        // [2][FS][LD]   phase 1
    bf16_t* Hs = reinterpret_cast<bf16_t*>(smem);          // [BM][LDH]     phase 2 (aliases phase-1 staging)
    bf16_t* W2s = Hs + BM * LDH;                           // [2][BN2][LDH] phase 2
    float* B1s = reinterpret_cast<float*>(smem + Cfg::kMain);   // [FS]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int split = blockIdx.x, nsplit = gridDim.x;
    const int m0 = blockIdx.y * BM, f0 = split * FS;

    for (int t = tid; t < FS; t += kFfnThreads) B1s[t] = b1 ? b1[f0 + t] : 0.0f;

    // ------------------------------ phase 1 -------------------------------------------
    {
        const int wf = wave >> 2, wm = wave & 3;
        f32x16 acc[FT][MT1];           // rows = hidden units, cols = rows of X
        zero_acc(acc);
        ActStager<BM> xa, xb;
        WeightStager<FS> wa, wb;
        const int nk = K / BK;                      // K % 64 == 0 (checked by the host)
        auto load = [&](ActStager<BM>& xs, WeightStager<FS>& ws, int kt) {
            xs.load(X, K, m0, kt * BK, M, tid);
            ws.load(W1, F, kt * BK, f0, tid);
        };
        auto tile = [&](int buf, bool store_next, const ActStager<BM>& xs, const WeightStager<FS>& ws) {
            const bf16_t* wsrc = W1s + buf * FS * LD;
            const bf16_t* asrc = Xs + (buf * BM + wm * MT1 * 32) * LD;
            // LDS latency under load is ~250 clocks, several MFMA groups long: fragments are fetched
            // D1 k-steps ahead of the matrix instructions that consume them.
            constexpr int D1 = 3;
            Frags<FT, MT1> fr[D1];
#pragma unroll
            for (int d = 0; d < D1; ++d) fr[d].fetch(wsrc, LD, wf * FT * 32, asrc, LD, d, i, h);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const Frags<FT, MT1> cur = fr[ks % D1];
                if (ks + D1 < 4) fr[ks % D1].fetch(wsrc, LD, wf * FT * 32, asrc, LD, ks + D1, i, h);
                if (store_next && ks == 0) xs.store(Xs + (buf ^ 1) * BM * LD, tid);
                if (store_next && ks == 1) ws.store(W1s + (buf ^ 1) * FS * LD, tid);
#pragma unroll
                for (int ft = 0; ft < FT; ++ft)
#pragma unroll
                    for (int mt = 0; mt < MT1; ++mt)
                        acc[ft][mt] = mfma32(cur.w[ft], cur.a[mt], acc[ft][mt]);
            }
        };
        // Tiles are processed in pairs so that the two register sets and the two LDS buffers have
        // fixed roles; prefetches past the end re-load the last tile (harmless) so that the loop
        // body is branch-free.
        load(xa, wa, 0);
        load(xb, wb, min(1, nk - 1));
        xa.store(Xs, tid);
        wa.store(W1s, tid);
        __syncthreads();
        int kt = 0;
        for (; kt + 1 < nk; kt += 2) {
            load(xa, wa, min(kt + 2, nk - 1));
            tile(0, true, xb, wb);
            __syncthreads();
            load(xb, wb, min(kt + 3, nk - 1));
            tile(1, true, xa, wa);
            __syncthreads();
        }
        if (kt < nk) {                      // odd tile count: the last tile sits in buffer 0
            tile(0, false, xb, wb);
            __syncthreads();
        }
        // epilogue: bias + activation, round to bf16, Hs[m][f] (f contiguous = phase-2 k)
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int fl = (wf * FT + ft) * 32 + 8 * g + 4 * h;   // local hidden index of 4 regs
                const float4 bv = *reinterpret_cast<const float4*>(B1s + fl);
#pragma unroll
                for (int mt = 0; mt < MT1; ++mt) {
                    const int ml = (wm * MT1 + mt) * 32 + i;
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
        const int wm = wave >> 2, wn = wave & 3;
        const bool full_block = m0 + BM <= M;       // uniform: no per-lane predication of the stores
        f32x16 acc[MT2][NT2];          // rows = rows of X, cols = output columns
        zero_acc(acc);
        typedef WeightStager<BN2, FS> W2Stager;     // one tile = the whole hidden slice x BN2 columns
        W2Stager wreg;                              // one register set: a tile is long enough to hide the loads
        const int T = K2 / BN2;                     // one tile per column block
        constexpr int KS = FS / 16;
        auto load = [&](W2Stager& ws, int nb) { ws.load(W2 + (long)f0 * K2, K2, 0, nb * BN2, tid); };
        auto tile = [&](int nb, int buf, bool store_next, const W2Stager& ws) {
            const bf16_t* wsrc = W2s + buf * BN2 * LDH;
            const bf16_t* asrc = Hs + (wm * MT2 * 32) * LDH;
            constexpr int D2 = KS < 4 ? KS : 4;
            Frags<NT2, MT2> fr[D2];
#pragma unroll
            for (int d = 0; d < D2; ++d) fr[d].fetch(wsrc, LDH, wn * NT2 * 32, asrc, LDH, d, i, h);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const Frags<NT2, MT2> cur = fr[ks % D2];
                if (ks + D2 < KS) fr[ks % D2].fetch(wsrc, LDH, wn * NT2 * 32, asrc, LDH, ks + D2, i, h);
                // the LDS stores of the next tile go late in this tile (its loads were issued at the
                // top of the tile), one unit per k step
#pragma unroll
                for (int u = 0; u < W2Stager::U; ++u)
                    if (store_next && ks == KS - 1 - (W2Stager::U - 1 - u)) ws.store_unit(W2s + (buf ^ 1) * BN2 * LDH, tid, u);
#pragma unroll
                for (int nt = 0; nt < NT2; ++nt)
#pragma unroll
                    for (int mt = 0; mt < MT2; ++mt)
                        acc[mt][nt] = mfma32(cur.a[mt], cur.w[nt], acc[mt][nt]);
            }
            {
                // this column block is complete: lane = output column, registers = rows of X
                // (32 lanes write 128 contiguous bytes of one row of the partial matrix).
                // 32-bit element offsets (the host checks nsplit * M * K2 < 2^31): one scalar multiply
                // and one vector add per store instead of 64-bit address arithmetic.
#pragma unroll
                for (int nt = 0; nt < NT2; ++nt) {
                    const unsigned col = nb * BN2 + (wn * NT2 + nt) * 32 + i;
                    const float bv = (nsplit == 1 && b2) ? b2[col] : 0.0f;
                    const unsigned row0 = m0 + wm * MT2 * 32 + 4 * h;
                    const unsigned base = ((nsplit == 1 ? 0u : (unsigned)split * (unsigned)M) + row0) * (unsigned)K2 + col;
#pragma unroll
                    for (int mt = 0; mt < MT2; ++mt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int dr = mt * 32 + 8 * (r >> 2) + (r & 3);      // compile-time row step
                            if (full_block || (int)row0 + dr < M) {
                                const unsigned idx = base + (unsigned)dr * (unsigned)K2;
                                if (nsplit == 1) Y[idx] = (bf16_t)(acc[mt][nt][r] + bv);
                                else part[idx] = acc[mt][nt][r];
                            }
                            acc[mt][nt][r] = 0.0f;
                        }
                }
            }
        };
        load(wreg, 0);
        wreg.store(W2s, tid);
        __syncthreads();       // also publishes Hs
        for (int nb = 0; nb < T; ++nb) {
            load(wreg, min(nb + 1, T - 1));          // past the end: re-load the last tile (never used)
            tile(nb, nb & 1, true, wreg);
            __syncthreads();
        }
    }
}

// y[m][n] = bf16( sum_s part[s][m][n] + b2[n] ), slices added in index order.
__global__ __launch_bounds__(256) void ffn_reduce_kernel(const float* __restrict__ part,
                                                         const float* __restrict__ b2,
                                                         bf16_t* __restrict__ Y, long MK2, int K2, int nsplit,
                                                         long slice_stride) {
    const long n4 = MK2 / 4;
    for (long i = blockIdx.x * 256L + threadIdx.x; i < n4; i += (long)gridDim.x * 256) {
        float4 a = reinterpret_cast<const float4*>(part)[i];
        for (int s = 1; s < nsplit; ++s) {
            const float4 v = reinterpret_cast<const float4*>(part + (long)s * slice_stride)[i];
            a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
        }
        if (b2) {
            const float4 bv = *reinterpret_cast<const float4*>(b2 + (int)((i * 4) % K2));
            a.x += bv.x; a.y += bv.y; a.z += bv.z; a.w += bv.w;
        }
        reinterpret_cast<uint2*>(Y)[i] = make_uint2(pack_bf16(a.x, a.y), pack_bf16(a.z, a.w));
    }
}

// slice_stride: elements between the partial results of consecutive slices (0: MK2, densely packed)
hipError_t ffn_reduce(const float* part, const float* b2, void* y, long MK2, int K2, int nsplit, hipStream_t s,
                      long slice_stride) {
    if (slice_stride == 0) slice_stride = MK2;
    long g = (MK2 / 4 + 255) / 256;
    if (g > 2048) g = 2048;
    hipLaunchKernelGGL(ffn_reduce_kernel, dim3((unsigned)g), dim3(256), 0, s, part, b2, (bf16_t*)y, MK2, K2, nsplit, slice_stride);
    return hipGetLastError();
}

template <int BM, int FS, int BN2>
static hipError_t launch_ffn(const void* x, const void* w1, const float* b1, const void* w2,
                             const float* b2, void* y, int M, int K, int F, int K2, int act,
                             void* workspace, hipStream_t s) {
    typedef FfnCfg<BM, FS, BN2> Cfg;
    auto kern = fused_ffn_kernel<BM, FS, BN2>;
    if (hipError_t e = allow_dynamic_lds<fused_ffn_kernel<BM, FS, BN2>>((int)((int)Cfg::kSmem)); e != hipSuccess) return e;
    const int nsplit = F / FS;
    dim3 grid(nsplit, (M + BM - 1) / BM);
    prof_start(2, s);
    prof_shape(2, grid.x * grid.y, kFfnThreads);
    hipLaunchKernelGGL(kern, grid, dim3(kFfnThreads), Cfg::kSmem, s, (const bf16_t*)x, (const bf16_t*)w1, b1,
                       (const bf16_t*)w2, b2, (bf16_t*)y, (float*)workspace, M, K, F, K2, act);
    hipError_t e = hipGetLastError();
    if (nsplit != 1) prof_mid(2, s);
    if (e == hipSuccess && nsplit != 1) e = ffn_reduce((const float*)workspace, b2, y, (long)M * K2, K2, nsplit, s);
    prof_stop(2, s);      // the event pair brackets the whole entry point, the reduction included
    return e;
}

// Tile configurations (BM rows, FS hidden slice, phase-2 column block BN2):
//   0: 128 x 192, 128   1: 128 x 128, 128   2: 128 x 64, 128
//   3: the wave-specialised streaming kernel (64 x 384, 384); the built-in choice whenever the
//      shape allows it (K % 64 == 0, F % 8 == 0, K2 % 8 == 0; the last hidden slice and the last
//      column block may be ragged)
//   4: the streaming kernel with four consumer waves of 64 x 96 wave tiles (64 x 384, 384), same shape rules
int fused_ffn_num_cfgs() { return 5; }

static bool ffn_cfg_ok(int cfg, int K, int F, int K2) {
    switch (cfg) {
        case 0: return F % 192 == 0 && K2 % 128 == 0;
        case 1: return F % 128 == 0 && K2 % 128 == 0;
        case 2: return F % 64 == 0 && K2 % 128 == 0;
        case 3: case 4: return fused_ffn_stream_ok(0, K, F, K2);
        default: return false;
    }
}

int fused_ffn_pick_cfg(int M, int K, int F, int K2, int tile_cfg) {
    (void)M;
    if (tile_cfg >= 0) return ffn_cfg_ok(tile_cfg, K, F, K2) ? tile_cfg : -1;
    if (ffn_cfg_ok(3, K, F, K2)) return 3;
    for (int c = 0; c < 3; ++c)
        if (ffn_cfg_ok(c, K, F, K2)) return c;
    return -1;
}

int fused_ffn_nsplit(int cfg, int F) {
    static const int fs[5] = {192, 128, 64, 384, 384};
    return (cfg >= 0 && cfg < 5) ? (F + fs[cfg] - 1) / fs[cfg] : 0;     // only the streaming kernels take ragged slices
}

hipError_t fused_ffn(const void* x, const void* w1, const float* b1, const void* w2, const float* b2,
                     void* y, int M, int K, int F, int K2, int act, int tile_cfg, void* workspace,
                     hipStream_t s) {
    switch (fused_ffn_pick_cfg(M, K, F, K2, tile_cfg)) {
        case 0: return launch_ffn<128, 192, 128>(x, w1, b1, w2, b2, y, M, K, F, K2, act, workspace, s);
        case 1: return launch_ffn<128, 128, 128>(x, w1, b1, w2, b2, y, M, K, F, K2, act, workspace, s);
        case 2: return launch_ffn<128, 64, 128>(x, w1, b1, w2, b2, y, M, K, F, K2, act, workspace, s);
        case 3: return fused_ffn_stream(x, w1, b1, w2, b2, y, M, K, F, K2, act, workspace, s);
        case 4: return fused_ffn_stream(x, w1, b1, w2, b2, y, M, K, F, K2, act, workspace, s, 1);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ago
