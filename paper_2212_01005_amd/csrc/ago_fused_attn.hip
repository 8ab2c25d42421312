// Fused matmul -> scale -> row softmax -> matmul (the attention chain of AGO Sec. VI-C;
// "downstream pointwise" rule of Sec. III-B: the downstream product keeps all of its output
// columns and consumes the upstream result in slices of its reduction dimension, the keys).
//
// One workgroup = 32 NQT query rows of one (batch, head), 2 NQT consumer waves and two producer waves.
//   consumer (qt, kh) owns the 32 query rows of tile qt and, of every 128-key block, the 64 keys
//       of half kh: the two waves of a query tile share a SIMD, so one's softmax arithmetic
//       overlaps the other's matrix instructions.  Each keeps its own running (max, sum, O^T); the
//       pair is merged once at the end through LDS.
//   producers (one for K, one for V): stream the blocks global -> LDS with the direct-to-LDS load
//       (no registers, no LDS stores, nothing transposed by hand), one block ahead, two LDS
//       buffers; they meet the consumers at one workgroup barrier per block.
// Per block and consumer:
//   S^T = K_blk Q^T         (rows = keys, cols = queries: a lane owns one query column, so the
//                            softmax statistics of a row are lane-local plus one cross-half step)
//   online softmax in fp32  (running max m and sum l per query, exp2 with scale*log2(e) folded in)
//   O^T += V_blk^T P^T      (P rounded to bf16; the accumulator layout of S^T *is* the B-operand
//                            layout of this product, so P never leaves registers; V^T fragments come
//                            from V's natural [key][d] layout through the transposing LDS read, whose
//                            row addresses also absorb the accumulator's key order)
// The scores and probabilities never leave the chip.
// LDS layouts (128-byte rows = one key; the producer realises the permutation by choosing which
// global 16-byte chunk each lane fetches): K chunk ^= (key >> 1) & 7; V chunk ^= bit 2 from key
// bit 1 and bit 1 from key bit 2.  Both make the fragment reads bank-conflict free.
#include "ago_dev.hpp"
#include "ago_launch.hpp"
#include "ago_host.hpp"

namespace ago {

constexpr int kD = 64;      // head-dimension columns per LDS plane (D = 64 NP)
constexpr int kKB = 128;    // keys per block
constexpr int kPlaneB = kKB * kD * 2;          // bytes of one 64-column plane of a K (or V) block: 16384

namespace {
typedef __attribute__((address_space(3))) unsigned char lds_byte;
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));

template <int N>
__device__ __forceinline__ void wait_vm() {
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}
__device__ __forceinline__ bf16x8 lds_read16(const lds_byte* p) {
    typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
    return *(const lds_bf16x8*)p;
}
// V^T fragment: rows = head-dimension columns (the lane offset encodes them), k = the 8 keys whose
// rows start at p (first four) and at p + 8 rows (last four)
__device__ __forceinline__ bf16x8 lds_read_vt(const lds_byte* p) {
    typedef __attribute__((address_space(3))) bf16x4_t lds_bf16x4;
    const bf16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p);
    const bf16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p + 8 * 128));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}
}  // namespace

// HAS_BIAS: an additive term between the scale and the softmax, Bias[b * bias_sb + hh * bias_sh + q * S + key]
// (a stride of 0 broadcasts over that dimension).  Each lane fetches the 32 values of its query row and
// its keys straight from global memory before the block's first product, so the loads overlap it.
// NP: 64-column planes of the head dimension (D = 64 NP).  A K or V block is stored plane by plane,
// [plane][128 keys][64], each plane with the layout described at the top, so every fragment address is
// the D = 64 one plus a plane offset.
template <int NQT, int NSTG, int BIAS /* 0 none, 1 rows by 16-byte loads, 2 element by element */, int NP = 1>
__global__ __launch_bounds__((2 * NQT + 2) * 64)
__attribute__((amdgpu_waves_per_eu(NP == 2 || BIAS == 2 ? 2 : (BIAS == 1 ? 4 : 3), 4))) void fused_attn_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    bf16_t* __restrict__ O, int S, int heads, int qblocks, int Hh, long stride_b, long stride_h, long stride_s,
    float c /* scale * log2(e) */, const bf16_t* __restrict__ Bias, long bias_sb, long bias_sh) {
    constexpr bool HAS_BIAS = BIAS != 0;
    constexpr int kBlockB = NP * kPlaneB;
    static_assert(NP == 1 || NSTG == 2, "two planes: two buffers");
    extern __shared__ __align__(16) unsigned char smem_generic[];
    lds_byte* smem = (lds_byte*)smem_generic;          // [2 buffers][K block | V block]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Workgroups are dealt round-robin to the 8 XCDs (one L2 each) in launch order: the query blocks
    // of one head get launch indices that are congruent modulo 8, so they land on the same XCD and
    // the head's K and V come from HBM once instead of once per query block.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int head = (slot / qblocks) * 8 + xcd, qblk = slot % qblocks;
    if (head >= heads) return;                         // padding workgroups of the last group of 8 heads
    // row s of (batch b, head hh) starts at b * stride_b + hh * stride_h + s * stride_s elements: the
    // [B][Hh][S][D] and [B][S][Hh][D] layouts (and any other with contiguous rows) without a transpose
    const long head_off = (long)(head / Hh) * stride_b + (long)(head % Hh) * stride_h;
    Q += head_off; K += head_off; V += head_off; O += head_off;
    const int nblk = (S + kKB - 1) / kKB;

    if (wave >= 2 * NQT) {
        // ================================ producers ========================================
        // Wave 2 NQT streams the K blocks, wave 2 NQT + 1 the V blocks.  Load q of a block covers its
        // rows 8 q .. 8 q + 7: lane = (row, physical chunk).  Keys beyond S are clamped to the last
        // key (their scores are masked by the consumers).
        const bool is_v = wave == 2 * NQT + 1;
        const bf16_t* src = is_v ? V : K;
        const int r8 = lane >> 3, pc = lane & 7;
        auto issue = [&](int blk) {
            lds_byte* dst = smem + (blk % NSTG) * 2 * kBlockB + (is_v ? kBlockB : 0);
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int row = 8 * q + r8;
                    const int sw = is_v ? ((((row >> 1) & 1) << 2) | (((row >> 2) & 1) << 1)) : ((row >> 1) & 7);
                    const bf16_t* g = src + (long)min(blk * kKB + row, S - 1) * stride_s + 64 * p + 8 * (pc ^ sw);
                    __builtin_amdgcn_global_load_lds((__attribute__((address_space(1))) const void*)g,
                                                     (__attribute__((address_space(3))) void*)(dst + p * kPlaneB + q * 1024), 16, 0, 0);
                }
        };
        auto wait_blocks = [&](int n) {      // at most n blocks (16 NP loads each) outstanding
            if (n >= 2) wait_vm<(NP == 1 ? 32 : 63)>();          // n = 2 only with three buffers, i.e. NP = 1
            else if (n == 1) wait_vm<16 * NP>();
            else wait_vm<0>();
        };
        static_assert(NSTG == 2 || NSTG == 3, "ring depth");
        const int npro = min(NSTG, nblk);
        for (int blk = 0; blk < npro; ++blk) issue(blk);
        wait_blocks(npro - 1);
        __builtin_amdgcn_s_barrier();                  // block 0 is in LDS
        for (int blk = 0; blk < nblk; ++blk) {
            // block blk + 1 must have landed before the consumers leave this iteration; blocks up to
            // blk + NSTG - 1 have been issued.  Block blk + NSTG can only be issued once the buffer of
            // block blk is free, i.e. after this iteration's barrier.
            wait_blocks(max(0, min(blk + NSTG - 1, nblk - 1) - (blk + 1)));
            __builtin_amdgcn_s_barrier();
            if (blk + NSTG < nblk) issue(blk + NSTG);
        }
        __builtin_amdgcn_s_barrier();                  // the consumers' merge barrier
        return;
    }

    // ================================== consumers ==========================================
    const int qt = wave % NQT, kh = wave / NQT;
    const int j = lane & 31, h = lane >> 5;
    const int q_row = qblk * (32 * NQT) + qt * 32 + j;

    bf16x8 qf[4 * NP];
#pragma unroll
    for (int ks = 0; ks < 4 * NP; ++ks)
        qf[ks] = __builtin_bit_cast(bf16x8, ld_u4(Q + (long)min(q_row, S - 1) * stride_s + ks * 16 + 8 * h));

    // K fragment of key tile kt (32 keys), k step ks: row = 64 kh + 32 kt + j, logical chunk 2 ks + h
    const int krow = 64 * kh + j;                      // + 32 kt: bit 5, does not reach the swizzle bits 1..3
    const int koff = krow * 128;
    const int ksw = (krow >> 1) & 7;
    // V^T fragment of (kt, u, dt): the lane addresses row (64 kh + 32 kt + 16 u + 4 h + (s >> 2)) [+ 8 for the
    // second read], head-dimension columns dt * 32 + 16 (g & 1) + 4 (s & 3) .. + 3
    const int g = lane >> 4, s15 = lane & 15;
    const int vrow0 = 64 * kh + 4 * h + (s15 >> 2);    // + 32 kt + 16 u (+ 8): bits 3..5; swizzle uses bits 1, 2
    const int vsw = (((vrow0 >> 1) & 1) << 2) | (((vrow0 >> 2) & 1) << 1);
    int voff[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt) {
        const int chunk = 4 * dt + 2 * (g & 1) + ((s15 & 3) >> 1);        // 16-byte chunk of the lane's 4 columns
        voff[dt] = vrow0 * 128 + ((chunk ^ vsw) << 4) + 8 * (s15 & 1);
    }

    f32x16 o[2 * NP];
#pragma unroll
    for (int dt = 0; dt < 2 * NP; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
    float m = -INFINITY, l = 0.f;     // running max of scaled scores, running (per-half) sum
    // with a bias the scores are rescaled (and biased) once, ahead of the max; without, the scale rides
    // in the exponent's multiply-add
    const float ce = HAS_BIAS ? 1.f : c;
    const bf16_t* brow = nullptr;
    if constexpr (HAS_BIAS)
        brow = Bias + (long)(head / Hh) * bias_sb + (long)(head % Hh) * bias_sh + (long)min(q_row, S - 1) * S;

    // Bias values of the lane's query row: register group gq of key tile kt covers the 4 consecutive
    // keys 4 h + 8 gq (+ 32 kt + 64 kh).  BIAS == 1 (S % 8 == 0, 16-byte aligned rows): lane (j, h) loads
    // the 8 keys 16 p + 8 h .. + 7 in one 16-byte access; its low half belongs to the h = 0 lane and its
    // high half to the h = 1 lane, so one swap of 32-lane halves per register pair (done when the values
    // are used) hands every lane its groups 2 p and 2 p + 1.  A chunk beyond S is clamped to the row's
    // last chunk (those keys are masked).  The loads are issued ahead of the block's first product; holding
    // them a whole iteration ahead would cost the 16 registers that separate 4 waves per SIMD from 3.
    uint4 bw[2][2];
    auto load_bias = [&](int blk) {
        const int key_wave = blk * kKB + 64 * kh;
        if constexpr (BIAS == 1) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int pr = 0; pr < 2; ++pr)
                    bw[kt][pr] = ld_u4(brow + min(key_wave + kt * 32 + 16 * pr + 8 * h, S - 8));
        } else {
            const unsigned short* be = reinterpret_cast<const unsigned short*>(brow);
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int pr = 0; pr < 2; ++pr) {
                    unsigned e8[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int key = key_wave + 4 * h + kt * 32 + 16 * pr + 8 * (e >> 2) + (e & 3);
                        e8[e] = be[min(key, S - 1)];
                    }
                    bw[kt][pr] = make_uint4(e8[0] | (e8[1] << 16), e8[2] | (e8[3] << 16), e8[4] | (e8[5] << 16),
                                            e8[6] | (e8[7] << 16));
                }
        }
    };
    __builtin_amdgcn_s_barrier();     // block 0 is in LDS
    for (int blk = 0; blk < nblk; ++blk) {
        const lds_byte* kb = smem + (blk % NSTG) * 2 * kBlockB;
        const lds_byte* vb = kb + kBlockB;

        if constexpr (HAS_BIAS) load_bias(blk);     // in flight across the first product

        f32x16 sc[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r) sc[kt][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4 * NP; ++ks)
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
                sc[kt] = mfma32(lds_read16(kb + (ks >> 2) * kPlaneB + koff + kt * 32 * 128 + (((2 * (ks & 3) + h) ^ ksw) << 4)),
                                qf[ks], sc[kt]);

        if constexpr (HAS_BIAS) {
            constexpr float kLog2e = 1.4426950408889634f;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int pr = 0; pr < 2; ++pr) {
                    uint4 w = bw[kt][pr];
                    if constexpr (BIAS == 1) {
                        const auto s0 = __builtin_amdgcn_permlane32_swap(w.x, w.z, false, false);
                        const auto s1 = __builtin_amdgcn_permlane32_swap(w.y, w.w, false, false);
                        w = make_uint4(s0[0], s1[0], s0[1], s1[1]);
                    }
                    const unsigned raw[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int r = 8 * pr + 2 * e;                  // registers r, r + 1 of key tile kt
                        sc[kt][r] = fmaf(sc[kt][r], c, __uint_as_float(raw[e] << 16) * kLog2e);
                        sc[kt][r + 1] = fmaf(sc[kt][r + 1], c, __uint_as_float(raw[e] & 0xffff0000u) * kLog2e);
                    }
                }
        }
        // mask keys beyond S (only a block that straddles S needs it; the test is wave-uniform)
        if ((blk + 1) * kKB > S) {
            const int key_base = blk * kKB + 64 * kh + 4 * h;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = key_base + kt * 32 + 8 * (r >> 2) + (r & 3);
                    sc[kt][r] = key < S ? sc[kt][r] : -INFINITY;
                }
        }
        // block max of the raw scores (c > 0 keeps the order); pairs fold into 3-input max
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int r = 0; r < 16; r += 2) mx = fmaxf(fmaxf(sc[kt][r], sc[kt][r + 1]), mx);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx * ce);
        // The reference m that the exponentials subtract only has to bound the scores from above loosely:
        // it moves (and the sum and O^T are rescaled, 16 (2 NP + ...) multiplies per lane) only when some
        // row of the wave saw its maximum grow by more than kLazy in the exponent, i.e. when staying put
        // would let a probability exceed 2^kLazy.  Any reference gives the same quotient at the end; after
        // the first block a new maximum that far above the old one is rare, so the rescale mostly
        // happens once.  (m = -inf, nothing seen yet: any finite maximum is "more".)
        constexpr float kLazy = 8.0f;
        if (__builtin_amdgcn_ballot_w64(m_new > m + kLazy) != 0) {        // wave-uniform
            // a half whose keys are all beyond S so far keeps m = -inf: subtract 0 instead (exp2(-inf) = 0)
            const float alpha = __builtin_amdgcn_exp2f(m - (m_new == -INFINITY ? 0.f : m_new));
            m = m_new;
            l *= alpha;
#pragma unroll
            for (int dt = 0; dt < 2 * NP; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
        }
        const float mref = m == -INFINITY ? 0.f : m;

        bf16x8 pf[2][2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float pv = __builtin_amdgcn_exp2f(fmaf(sc[kt][8 * u + e], ce, -mref));
                    l += pv;
                    pf[kt][u][e] = (bf16_t)pv;
                }
        // the lane's two V^T base addresses of this block, once: the 8 NP fragment addresses are these plus constants
        const lds_byte* vbase[2] = {vb + voff[0], vb + voff[1]};
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int dt = 0; dt < 2 * NP; ++dt)
                    o[dt] = mfma32(lds_read_vt(vbase[dt & 1] + (dt >> 1) * kPlaneB + (kt * 32 + 16 * u) * 128), pf[kt][u], o[dt]);

        __builtin_amdgcn_s_barrier();
    }

    // merge the two key halves of each query tile, both waves at work: wave kh finishes the NP output
    // tiles dt = kh NP .. kh NP + NP - 1 (32 head-dimension columns each).  It parks (m, l) and the tiles
    // the other wave finishes in LDS (the K / V buffers are free after the last barrier), and after one
    // barrier combines its own tiles with what the other parked and writes them.
    l += __shfl_xor(l, 32, 64);
    constexpr int kParkRows = 2 + 16 * NP;             // m, l, 16 NP accumulator registers
    float* park = reinterpret_cast<float*>(smem_generic) + (qt * 2 + kh) * kParkRows * 64;      // [tile][kh][rows][64]
    const float* theirs = reinterpret_cast<const float*>(smem_generic) + (qt * 2 + (kh ^ 1)) * kParkRows * 64;
    park[lane] = m;
    park[64 + lane] = l;
#pragma unroll
    for (int t = 0; t < NP; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            // kh is wave-uniform: select the register of the tile the other wave owns without dynamic indexing
            const float mine_low = o[t][r], mine_high = o[NP + t][r];
            park[(2 + t * 16 + r) * 64 + lane] = kh == 0 ? mine_high : mine_low;
        }
    __syncthreads();
    {
        const float m1 = theirs[lane], l1 = theirs[64 + lane];
        const float mt = fmaxf(m, m1);                 // finite unless a bias of -inf covers the whole row
        const float a0 = __builtin_amdgcn_exp2f(m - mt), a1 = __builtin_amdgcn_exp2f(m1 - mt);
        const float inv = 1.0f / (l * a0 + l1 * a1);
        const float w0 = a0 * inv, w1 = a1 * inv;
#pragma unroll
        for (int t = 0; t < NP; ++t) {
            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[r] = (kh == 0 ? o[t][r] : o[NP + t][r]) * w0 + theirs[(2 + t * 16 + r) * 64 + lane] * w1;
            if (q_row < S) {
                const int dt = kh * NP + t;
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int d = dt * 32 + 8 * gq + 4 * h;
                    *reinterpret_cast<uint2*>(O + (long)q_row * stride_s + d) =
                        make_uint2(pack_bf16(acc[4 * gq], acc[4 * gq + 1]), pack_bf16(acc[4 * gq + 2], acc[4 * gq + 3]));
                }
            }
        }
    }
}

struct AttnBias {
    const void* ptr;
    long sb, sh;      // element strides over batch and head, 0 = broadcast
};

template <int NQT, int NSTG, int BIAS, int NP = 1>
static hipError_t launch_attn(const void* q, const void* k, const void* v, void* o, int B, int Hh, int S,
                              long stride_b, long stride_h, long stride_s, float scale, hipStream_t s,
                              AttnBias bias = AttnBias{nullptr, 0, 0}) {
    constexpr size_t smem = (size_t)NSTG * 2 * NP * kPlaneB;    // ring of (K block, V block) buffers; the merge reuses them
    static_assert((size_t)NQT * (2 + 32 * NP) * 64 * 4 <= smem, "merge scratch");
    auto kern = fused_attn_kernel<NQT, NSTG, BIAS, NP>;
    if (hipError_t e = allow_dynamic_lds<fused_attn_kernel<NQT, NSTG, BIAS, NP>>((int)((int)smem)); e != hipSuccess) return e;
    const int heads = B * Hh, qblocks = (S + 32 * NQT - 1) / (32 * NQT);
    dim3 grid((unsigned)(8 * qblocks * ((heads + 7) / 8)));
    prof_start(3, s);
    prof_shape(3, grid.x, (2 * NQT + 2) * 64);
    hipLaunchKernelGGL(kern, grid, dim3((2 * NQT + 2) * 64), smem, s, (const bf16_t*)q, (const bf16_t*)k,
                       (const bf16_t*)v, (bf16_t*)o, S, heads, qblocks, Hh, stride_b, stride_h, stride_s,
                       scale * 1.4426950408889634f, (const bf16_t*)bias.ptr, bias.sb, bias.sh);
    prof_stop(3, s);
    return hipGetLastError();
}

// Tile configurations: query rows per workgroup (two workgroups share a compute unit except for 3).
//   0: 96   1: 128   2: 64   3: 192, one workgroup per compute unit, three LDS buffers
int fused_attn_num_cfgs() { return 4; }

hipError_t fused_attn(const void* q, const void* k, const void* v, void* o, int B, int Hh, int S,
                      float scale, int tile_cfg, hipStream_t s, long stride_b, long stride_h, long stride_s, int D) {
    if (stride_s == 0) { stride_b = (long)Hh * S * D; stride_h = (long)S * D; stride_s = D; }   // [B][Hh][S][D]
    if (D == 128) {
        // two planes: 96 queries per workgroup (eight waves, two per SIMD: 32 query-fragment, 64 output and
        // 32 score registers per lane need that budget), 64 for configuration 2
        if (tile_cfg == 2) return launch_attn<2, 2, 0, 2>(q, k, v, o, B, Hh, S, stride_b, stride_h, stride_s, scale, s);
        return launch_attn<3, 2, 0, 2>(q, k, v, o, B, Hh, S, stride_b, stride_h, stride_s, scale, s);
    }
    if (D != 64) return hipErrorInvalidValue;
    if (tile_cfg < 0) {        // built-in choice: the candidate the time model predicts fastest
        AttnPlan plan;
        tile_cfg = plan_attn(B, Hh, S, 64, -1, &plan) ? plan.cfg : 0;
    }
    switch (tile_cfg) {
        case 1: return launch_attn<4, 2, 0>(q, k, v, o, B, Hh, S, stride_b, stride_h, stride_s, scale, s);
        case 2: return launch_attn<2, 2, 0>(q, k, v, o, B, Hh, S, stride_b, stride_h, stride_s, scale, s);
        case 3: return launch_attn<6, 3, 0>(q, k, v, o, B, Hh, S, stride_b, stride_h, stride_s, scale, s);
        default: return launch_attn<3, 2, 0>(q, k, v, o, B, Hh, S, stride_b, stride_h, stride_s, scale, s);
    }
}

// The chain with an additive bias / mask ahead of the softmax; q, k, v, o contiguous [B][Hh][S][D].
hipError_t fused_attn_bias(const void* q, const void* k, const void* v, const void* bias, void* o, int B, int Hh,
                           int S, long bias_sb, long bias_sh, float scale, int tile_cfg, hipStream_t s, int D) {
    const long stride_b = (long)Hh * S * D, stride_h = (long)S * D, stride_s = D;
    const AttnBias bs{bias, bias_sb, bias_sh};
    // Two LDS buffers throughout (the third costs the registers that the bias values need); the
    // element-by-element variant needs more registers still and runs configuration 3 as configuration 1.
    if (tile_cfg < 0) {
        AttnPlan plan;
        tile_cfg = plan_attn(B, Hh, S, 64, -1, &plan) ? plan.cfg : 0;
    }
    // 16-byte loads of 8 bias values need every row start 16-byte aligned
    const bool vec = S % 8 == 0 && bias_sb % 8 == 0 && bias_sh % 8 == 0 && reinterpret_cast<uintptr_t>(bias) % 16 == 0;
    if (D == 128) {
        if (vec) return launch_attn<3, 2, 1, 2>(q, k, v, o, B, Hh, S, stride_b, stride_h, stride_s, scale, s, bs);
        return launch_attn<3, 2, 2, 2>(q, k, v, o, B, Hh, S, stride_b, stride_h, stride_s, scale, s, bs);
    }
    if (D != 64) return hipErrorInvalidValue;
#define AGO_ATTN_BIAS_CASE(NQT, NQT_E)                                                                        \
    return vec ? launch_attn<NQT, 2, 1>(q, k, v, o, B, Hh, S, stride_b, stride_h, stride_s, scale, s, bs)     \
               : launch_attn<NQT_E, 2, 2>(q, k, v, o, B, Hh, S, stride_b, stride_h, stride_s, scale, s, bs)
    switch (tile_cfg) {
        case 1: AGO_ATTN_BIAS_CASE(4, 4);
        case 2: AGO_ATTN_BIAS_CASE(2, 2);
        case 3: AGO_ATTN_BIAS_CASE(6, 4);
        default: AGO_ATTN_BIAS_CASE(3, 3);
    }
#undef AGO_ATTN_BIAS_CASE
}

}  // namespace ago
