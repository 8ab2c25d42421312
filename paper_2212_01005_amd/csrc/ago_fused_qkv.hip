// Sibling fusion (AGO Sec. III: operators that share an input belong to one subgraph): the query, key
// and value projections of an attention layer as one kernel,
//   q = x Wq + bq,  k = x Wk + bk,  v = x Wv + bv,       x:[B*S][K], W*:[K][Hh*D]
// with the transpose that follows them ([B][S][Hh][D] -> [B][Hh][S][D]) folded into the store addresses.
//
// The launch covers the concatenated column space [q | k | v]: column block bx belongs to sibling
// bx / nb (nb = blocks per sibling) and picks that sibling's weight, bias and output pointers, so the
// three products are one grid, one pass over x through L2, and no separate transpose kernels.
// Tile 128 x 128 per workgroup (2 x 2 waves, each 64 x 64 on the 32x32x16 bf16 matrix instruction),
// K step 64, double-buffered LDS, weights transposed [K][N] -> [N][K] in registers on the way in.
#include "ago_dev.hpp"
#include "ago_launch.hpp"

namespace ago {

struct QkvParams {
    const bf16_t* x;
    const bf16_t* w[3];
    const float* b[3];
    bf16_t* o[3];
    int M, K, N;        // rows B*S, reduction, columns Hh*D of each sibling
    int S, Hh, D;
    int nb;             // column blocks per sibling
    int head_major;     // 1: o[b][hh][s][d]   0: o[b][s][hh][d] (= [M][N])
};

__global__ __launch_bounds__(256) void fused_qkv_kernel(const QkvParams p) {
    constexpr int BM = 128, BN = 128, BK = 64, LD = BK + 8, MT = 2, NT = 2;
    constexpr int A_CH = BM * BK / 8 / 256;          // 16-byte chunks of x per thread
    constexpr int BT_U = (BK / 8) * (BN / 4) / 256;  // 8x4 transpose units of a [K][N] weight tile per thread
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* As = reinterpret_cast<bf16_t*>(smem);    // [2][BM][LD]
    bf16_t* Bs = As + 2 * BM * LD;                   // [2][BN][LD]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int which = blockIdx.x / p.nb;             // sibling: 0 q, 1 k, 2 v
    const int m0 = blockIdx.y * BM, n0 = (blockIdx.x % p.nb) * BN;
    const bf16_t* A = p.x;
    const bf16_t* B = p.w[which];
    const int M = p.M, K = p.K, N = p.N;

    uint4 ra[A_CH];
    uint2 rbt[BT_U][8];
    auto load_tile = [&](int k0) {
#pragma unroll
        for (int u = 0; u < A_CH; ++u) {
            const int c = tid + 256 * u, row = c / (BK / 8), kc = c % (BK / 8);
            const int gm = m0 + row, gk = k0 + kc * 8;
            ra[u] = (gm < M && gk < K) ? ld_u4(A + (long)gm * K + gk) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < BT_U; ++u) {
            const int c = tid + 256 * u, nq = c % (BN / 4), ko = c / (BN / 4);
            const int gn = n0 + nq * 4;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const int gk = k0 + ko * 8 + kk;
                rbt[u][kk] = (gn < N && gk < K) ? *reinterpret_cast<const uint2*>(B + (long)gk * N + gn)
                                                : make_uint2(0, 0);
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
#pragma unroll
        for (int u = 0; u < BT_U; ++u) {
            const int c = tid + 256 * u, nq = c % (BN / 4), ko = c / (BN / 4);
            uint4 t[4];
            transpose_8x4(rbt[u], t);
#pragma unroll
            for (int q = 0; q < 4; ++q) st_u4(bs + (nq * 4 + q) * LD + ko * 8, t[q]);
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

    // epilogue: a lane holds column j of each 32 x 32 tile (16 rows); 32 lanes = 32 consecutive d of one head
    const int j = lane & 31, h = lane >> 5;
    const float* bias = p.b[which];
    bf16_t* O = p.o[which];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int col = n0 + (wn * NT + n) * 32 + j;
        if (col >= N) continue;
        const float bv = bias ? bias[col] : 0.0f;
        const int hh = col / p.D, d = col % p.D;
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + (wm * MT + m) * 32 + acc_row(r, h);
                if (row >= M) continue;
                long off = (long)row * N + col;
                if (p.head_major) {
                    const int bi = row / p.S, s = row % p.S;
                    off = (((long)bi * p.Hh + hh) * p.S + s) * p.D + d;
                }
                O[off] = (bf16_t)(acc[m][n][r] + bv);
            }
    }
}

hipError_t fused_qkv(const void* x, const void* wq, const void* wk, const void* wv, const float* bq,
                     const float* bk, const float* bv, void* q, void* k, void* v, int B, int S, int K, int Hh,
                     int D, int head_major, hipStream_t s) {
    QkvParams p;
    p.x = (const bf16_t*)x;
    p.w[0] = (const bf16_t*)wq; p.w[1] = (const bf16_t*)wk; p.w[2] = (const bf16_t*)wv;
    p.b[0] = bq; p.b[1] = bk; p.b[2] = bv;
    p.o[0] = (bf16_t*)q; p.o[1] = (bf16_t*)k; p.o[2] = (bf16_t*)v;
    p.M = B * S; p.K = K; p.N = Hh * D; p.S = S; p.Hh = Hh; p.D = D;
    p.nb = (p.N + 127) / 128;
    p.head_major = head_major;
    constexpr size_t smem = (size_t)2 * (128 + 128) * (64 + 8) * sizeof(bf16_t);
    if (hipError_t e = allow_dynamic_lds<fused_qkv_kernel>((int)smem); e != hipSuccess) return e;
    dim3 grid((unsigned)(3 * p.nb), (unsigned)((p.M + 127) / 128));
    hipLaunchKernelGGL(fused_qkv_kernel, grid, dim3(256), smem, s, p);
    return hipGetLastError();
}

}  // namespace ago
