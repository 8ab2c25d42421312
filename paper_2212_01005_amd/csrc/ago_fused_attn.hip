// Fused matmul -> scale -> row softmax -> matmul (the attention chain of AGO Sec. VI-C;
// "downstream pointwise" rule of Sec. III-B: the downstream product keeps all of its output
// columns and consumes the upstream result in slices of its reduction dimension, the keys).
//
// One workgroup = 4 waves = 128 query rows of one (batch, head); each wave owns 32 query rows.
// Keys / values are streamed through LDS in blocks of 128 with register prefetch.  Per block:
//   S^T = K_blk Q^T         (rows = keys, cols = queries: a lane owns one query column, so the
//                            softmax statistics of a row are lane-local plus one cross-half step)
//   online softmax in fp32  (running max m and sum l per query, exp2 with scale*log2(e) folded in)
//   O^T += V_blk^T P^T      (P rounded to bf16; the accumulator layout of S^T *is* the B-operand
//                            layout of this product, so P never leaves registers)
// The scores and probabilities never leave the chip.  V is transposed while it is staged into
// LDS, with the keys of every group of 16 permuted to match the accumulator row order.
#include "ago_dev.hpp"
#include "ago_launch.hpp"

namespace ago {

constexpr int kD = 64;      // head dimension
constexpr int kKB = 128;    // keys per block

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void fused_attn_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    bf16_t* __restrict__ O, int S, float c /* scale * log2(e) */) {
    constexpr int LDK = kD + 8, LDV = kKB + 8;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t (*Ks)[kKB][LDK] = reinterpret_cast<bf16_t (*)[kKB][LDK]>(smem);                       // [2]
    bf16_t (*Vt)[kD][LDV] = reinterpret_cast<bf16_t (*)[kD][LDV]>(smem + 2 * kKB * LDK * 2);     // [2]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 31, h = lane >> 5;
    const long head_off = (long)blockIdx.y * S * kD;
    Q += head_off; K += head_off; V += head_off; O += head_off;
    const int q_row = blockIdx.x * 128 + wave * 32 + j;

    bf16x8 qf[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        uint4 v = make_uint4(0, 0, 0, 0);
        v = ld_u4(Q + (long)min(q_row, S - 1) * kD + ks * 16 + 8 * h);
        qf[ks] = __builtin_bit_cast(bf16x8, v);
    }

    uint4 rk[4];
    uint2 rv[8];
    // Keys beyond S are clamped to the last key: their scores are masked to -inf below, so their
    // probabilities are exactly 0 and the (finite) duplicate K / V rows contribute nothing.
    // Unpredicated loads keep the block loop free of branches.
    auto load_block = [&](int key0) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int cidx = tid + 256 * u, row = cidx >> 3, kc = cidx & 7;
            rk[u] = ld_u4(K + (long)min(key0 + row, S - 1) * kD + kc * 8);
        }
        const int nq = tid & 15, ko = tid >> 4;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
            rv[kk] = *reinterpret_cast<const uint2*>(V + (long)min(key0 + ko * 8 + kk, S - 1) * kD + nq * 4);
    };
    auto store_block = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int cidx = tid + 256 * u, row = cidx >> 3, kc = cidx & 7;
            st_u4(&Ks[buf][row][kc * 8], rk[u]);
        }
        const int nq = tid & 15, ko = tid >> 4;
        uint4 t[4];
        transpose_8x4(rv, t);
        // keys ko*8 .. ko*8+7 of a group of 16: first four -> positions 4*(ko&1).., last four ->
        // positions 8 + 4*(ko&1)..  (lane half h of the matrix instruction reads positions 8h..8h+7)
        const int gb = (ko >> 1) * 16 + 4 * (ko & 1);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            *reinterpret_cast<uint2*>(&Vt[buf][nq * 4 + q][gb]) = make_uint2(t[q].x, t[q].y);
            *reinterpret_cast<uint2*>(&Vt[buf][nq * 4 + q][gb + 8]) = make_uint2(t[q].z, t[q].w);
        }
    };

    f32x16 o[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) { o[0][r] = 0.f; o[1][r] = 0.f; }
    float m = -INFINITY, l = 0.f;     // running max of scaled scores, running (per-half) sum

    const int nblk = (S + kKB - 1) / kKB;
    load_block(0);
    store_block(0);
    __syncthreads();
    for (int blk = 0; blk < nblk; ++blk) {
        const int buf = blk & 1;
        load_block(min(blk + 1, nblk - 1) * kKB);     // past the end: re-load the last block

        f32x16 s[4];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
                s[kt] = mfma32(ld_bf16x8(&Ks[buf][kt * 32 + j][ks * 16 + 8 * h]), qf[ks], s[kt]);

        // mask keys beyond S (only a block that straddles S needs it; the test is wave-uniform)
        if ((blk + 1) * kKB > S) {
            const int key_base = blk * kKB + 4 * h;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = key_base + kt * 32 + 8 * (r >> 2) + (r & 3);
                    s[kt][r] = key < S ? s[kt][r] : -INFINITY;
                }
        }
        // block max of the raw scores (c > 0 keeps the order); pairs fold into 3-input max
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int r = 0; r < 16; r += 2) mx = fmaxf(fmaxf(s[kt][r], s[kt][r + 1]), mx);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx * c);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        l *= alpha;
#pragma unroll
        for (int r = 0; r < 16; ++r) { o[0][r] *= alpha; o[1][r] *= alpha; }

        bf16x8 pf[4][2];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float pv = __builtin_amdgcn_exp2f(fmaf(s[kt][8 * u + e], c, -m_new));
                    l += pv;
                    pf[kt][u][e] = (bf16_t)pv;
                }
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
                    o[dt] = mfma32(ld_bf16x8(&Vt[buf][dt * 32 + j][kt * 32 + 16 * u + 8 * h]), pf[kt][u], o[dt]);

        store_block(buf ^ 1);
        __syncthreads();
    }

    l += __shfl_xor(l, 32, 64);
    const float inv = 1.0f / l;
    if (q_row < S) {
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int d = dt * 32 + 8 * g + 4 * h;
                *reinterpret_cast<uint2*>(O + (long)q_row * kD + d) =
                    make_uint2(pack_bf16(o[dt][4 * g] * inv, o[dt][4 * g + 1] * inv),
                               pack_bf16(o[dt][4 * g + 2] * inv, o[dt][4 * g + 3] * inv));
            }
    }
}

int fused_attn_num_cfgs() { return 1; }

hipError_t fused_attn(const void* q, const void* k, const void* v, void* o, int B, int Hh, int S,
                      float scale, int tile_cfg, hipStream_t s) {
    (void)tile_cfg;
    constexpr size_t smem = (size_t)2 * kKB * (kD + 8) * 2 + (size_t)2 * kD * (kKB + 8) * 2;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fused_attn_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((S + 127) / 128, (unsigned)(B * Hh));
    prof_start(3, s);
    hipLaunchKernelGGL(fused_attn_kernel, grid, dim3(256), smem, s, (const bf16_t*)q, (const bf16_t*)k,
                       (const bf16_t*)v, (bf16_t*)o, S, scale * 1.4426950408889634f);
    prof_stop(3, s);
    return hipGetLastError();
}

}  // namespace ago
