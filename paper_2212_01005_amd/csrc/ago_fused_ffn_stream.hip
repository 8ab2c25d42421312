// Fused matmul -> activation -> matmul, wave-specialised streaming variant (pw->pw, the
// "downstream pointwise" rule of AGO Sec. III-B / Fig. 7b: the downstream tile keeps all of its
// output channels, the upstream tile is a slice of the hidden dimension).
//
// Workgroup (split s, row block rb) owns 64 rows of X and 384 hidden units.  Twelve waves:
//   waves 0..7   consumers: LDS -> MFMA only (plus the two epilogues)
//   waves 8..11  producers: global -> LDS only, with the direct-to-LDS load (no registers, no LDS
//                store instructions); weights land in their natural [k][n] layout and the consumers
//                read them with the transposing LDS read, so nothing is transposed by hand.
//                Three of them stream weight tiles, the fourth streams X far ahead (see below)
// The two kinds of wave meet at one workgroup barrier per 32-deep k-tile.  Tiles travel through a
// ring of four LDS stages: during iteration t the producers issue tile t+3 and wait until tile
// t+2 has landed, the consumers multiply tile t and already fetch the fragments of tile t+1, so
// neither the global latency nor the LDS latency is exposed at a barrier.
//   phase 1  Hs[64][384] = act(X[rb] W1[:, slice] + b1[slice])      K/32 tiles of X and W1
//   phase 2  P[s][rb]    = Hs W2[slice, :]                          12 tiles of W2 per 384 columns
// The F/384 partial products are summed by ffn_reduce (which adds b2 and rounds); with a single
// slice phase 2 writes y directly.
//
// LDS layouts (16-byte chunks; the producers realise the permutation by choosing which global
// chunk each lane fetches, because the direct load writes lane i's 16 bytes at base + 16 i):
//   X block  [64 m][64 k] (two tiles): 128-byte rows, chunk ^= (m >> 1) & 7
//   W tile   [32 k][384 n]: 768-byte rows, 32-byte chunk pair ^= ((k & 3) << 1) | ((k >> 3) & 1)
//   Hs       [64 m][384 f] bf16, 392 elements per row
// All three give conflict-free fragment reads.
//
// Template parameters: MW 32-row tiles per consumer wave, BK tile depth, CW consumer waves (4 column
// groups x CW / 4 row groups; rows per workgroup = 32 MW CW / 4).  Two instantiations are launched, both
// with 64 rows per workgroup: <1, 32, 8> (eight consumer waves, 32 x 96 wave tiles: 7 LDS reads per 3
// matrix instructions and k step) and <2, 32, 4> (four consumer waves, 64 x 96 wave tiles: 8 reads per 6
// matrix instructions, one consumer wave per SIMD, 239 registers).  They run within 2% of each other,
// i.e. the consumers' LDS read issue is not what bounds the kernel; the first is the default.  A
// 128-row workgroup (<2, 16, 8>, half the L2 -> LDS traffic per FLOP) needs about 200 registers per lane
// with twelve waves per workgroup, 30 more than three waves per SIMD leave, and is not instantiated.
#include "ago_dev.hpp"
#include "ago_launch.hpp"
#include <type_traits>

namespace ago {
namespace {

constexpr int kProducerWaves = 4;
constexpr int FS = 384, CB = 384;
constexpr int kRowB = 384 * 2;                 // bytes per k-row of a weight tile
constexpr int kWWaves = kProducerWaves - 1;    // three waves load weights, one loads X
constexpr int kXRing = 4096;
constexpr int kHsLd = FS + 8;

// MW: 32-row tiles per consumer wave; BK_: tile depth; CW: consumer waves (4 column groups x CW / 4 row groups)
template <int MW, int BK_, int CW>
struct StreamCfg {
    static constexpr int kThreads = (CW + kProducerWaves) * 64;
    static constexpr int WMG = CW / 4;                      // row groups of consumer waves
    static constexpr int BM = 32 * MW * WMG, BK = BK_;
    static constexpr int KSTEPS = BK / 16;                  // 16-deep k steps per tile
    static constexpr int NST = 98304 / (BK * kRowB);        // ring stages: 96 KB of weight tiles (4 or 8)
    static constexpr int DIST = NST - 1;                    // tiles a producer runs ahead of the consumers
    static constexpr int TPB = 64 / BK;                     // tiles per 64-deep X block
    static constexpr int kXBlockB = BM * 64 * 2;            // X travels in 64-deep blocks (whole 128-byte lines)
    static constexpr int kXLoads = kXBlockB / 1024;         // direct loads of 1 KB per X block: 8 or 16
    static constexpr int kXLead = BM == 64 ? 4 : 3;         // X blocks in flight ahead (at most 63 loads outstanding)
    static constexpr int kXSlots = BM == 64 ? 7 : 5;
    static constexpr int kWTileB = BK * kRowB;              // 24576 or 12288
    static constexpr int kHsB = BM * kHsLd * 2;             // 50176 or 100352
    // Hs is only written after the last phase-1 tile has been consumed, so the phase-1 buffers may
    // overlap it; the phase-2 ring starts right behind Hs.
    static constexpr int kRing1 = kXRing + kXSlots * kXBlockB;
    static constexpr int kRing2 = kHsB;
    static constexpr int kB1 = 159744;
    static constexpr int kSmem = kB1 + FS * 4;              // 161280
    static constexpr int kWLoadsPerWave = kWTileB / 1024 / kWWaves;      // 8 or 4 direct loads per wave and tile
    static_assert((NST & (NST - 1)) == 0 && kRing1 + NST * kWTileB <= kB1, "phase-1 rings must not reach the bias slice");
    static_assert(kRing2 + NST * kWTileB <= kB1, "phase-2 ring must not reach the bias slice");
    static_assert(kSmem <= 160 * 1024, "LDS");
    static_assert(kXSlots >= kXLead + 1 && kXLead * kXLoads < 64, "X ring");
    static_assert(kWLoadsPerWave * 1024 * kWWaves == kWTileB, "weight tile split over the producer waves");
};

typedef __attribute__((address_space(3))) unsigned char lds_byte;
typedef __attribute__((address_space(1))) const void gptr_t;
typedef __attribute__((address_space(3))) void lptr_t;
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));

// wait until at most n of this wave's vector-memory operations are outstanding (n < 64)
template <int N>
__device__ __forceinline__ void wait_vm() {
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// 16 bytes per lane from global memory straight into LDS at base + 16 * lane (base wave-uniform)
__device__ __forceinline__ void load_to_lds(const bf16_t* src, lds_byte* base) {
    __builtin_amdgcn_global_load_lds((gptr_t*)src, (lptr_t*)base, 16, 0, 0);
}

// fragment of a weight tile for the 32 columns starting at the column pair the lane offset encodes:
// two transposing reads (k rows 0..3 and 4..7 of the lane's k-group)
__device__ __forceinline__ bf16x8 read_w_frag(const lds_byte* p) {
    typedef __attribute__((address_space(3))) bf16x4_t lds_bf16x4;
    const bf16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p));
    const bf16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p + 4 * kRowB));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}
__device__ __forceinline__ bf16x8 read_a_frag(const lds_byte* p) {
    typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
    return *(const lds_bf16x8*)p;
}

template <int MW>
struct Frag {
    bf16x8 a[MW], w[3];
};

// RAGGED: F or K2 is not a multiple of 384 (the exact instantiation carries none of the clamps and masks)
template <int MW, int BK_, int CW, bool RAGGED>
__global__ __launch_bounds__((CW + kProducerWaves) * 64) void fused_ffn_stream_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ W1, const float* __restrict__ b1,
    const bf16_t* __restrict__ W2, const float* __restrict__ b2, bf16_t* __restrict__ Y,
    float* __restrict__ part, int M, int K, int F, int K2, int act) {
    extern __shared__ __align__(16) unsigned char smem_generic[];
    lds_byte* smem = (lds_byte*)smem_generic;
    const int tid0 = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);
    typedef StreamCfg<MW, BK_, CW> C;
    constexpr int kConsumerWaves = CW, WMG = C::WMG;
    constexpr int BM = C::BM, BK = C::BK, KSTEPS = C::KSTEPS, TPB = C::TPB;
    constexpr int kXBlockB = C::kXBlockB, kXSlots = C::kXSlots, kXLead = C::kXLead, kXLoads = C::kXLoads;
    constexpr int kWTileB = C::kWTileB, kRing1 = C::kRing1, kRing2 = C::kRing2, kB1 = C::kB1;
    constexpr int kWLoadsPerWave = C::kWLoadsPerWave, NST = C::NST, DIST = C::DIST;
    const int split = blockIdx.x, nsplit = gridDim.x;
    const int f0 = split * FS;
    const int nrb = (M + BM - 1) / BM;       // row blocks; a workgroup walks blockIdx.y, blockIdx.y + gridDim.y, ...
    const int NT1 = K / BK;                 // phase-1 tiles
    const int NCB = (K2 + CB - 1) / CB;     // phase-2 column blocks (the last one may be ragged)
    // The last hidden slice may be ragged too (F and K2 are multiples of 8, one 16-byte chunk).  The
    // producers clamp what they fetch beyond F / K2 to valid addresses; the hidden units beyond F are
    // written as 0 into Hs, so whatever W2 rows stand in for them contribute nothing, and columns
    // beyond K2 are never stored.
    const int fvalid = RAGGED ? min(FS, F - f0) : FS;     // hidden units of this slice that exist
    const int NT2 = NCB * (FS / BK);        // phase-2 tiles
    // The workgroups of one hidden slice run in lockstep on one XCD and would all ask its L2 for the
    // same lines at the same moment (and W1's row stride maps a tile onto few L2 channels): each row
    // block walks the reduction dimension from a different starting tile instead.
    // (the phase-1 rotation is a whole number of X blocks)
    // Every pass of this loop is one row block, start to finish, with the same number of workgroup
    // barriers for every wave; the next pass's first loads only overwrite LDS that the previous pass has
    // finished reading before its last barrier.
    for (int rb = blockIdx.y; rb < nrb; rb += gridDim.y) {
    // opaque copy of the thread id: keeps the per-lane offsets of a pass from being hoisted out of this
    // loop and held in registers across the whole kernel
    int tid = tid0;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int m0 = rb * BM;
    const int rot1 = TPB * (rb % (NT1 / TPB)), rot2 = rb % (FS / BK);

    if (wave >= kConsumerWaves) {
        // ================================ producers ======================================
        const int pw = wave - kConsumerWaves;
        if (pw == kWWaves) {
            // ---- the X wave.  Every row block reads its own rows of X, so these loads miss the L2
            // that serves the (shared) weight tiles and take much longer; loads complete in order
            // within a wave, hence a wave of their own, running kXLead blocks (2 kXLead tiles) ahead.
            unsigned xoff[kXLoads];           // load q: rows 8 q .. 8 q + 7 x 128 bytes; lane = (row, physical chunk)
#pragma unroll
            for (int q = 0; q < kXLoads; ++q) {
                const int xrow = 8 * q + (lane >> 3);
                const int xchunk = (lane & 7) ^ ((xrow >> 1) & 7);
                xoff[q] = (unsigned)min(m0 + xrow, M - 1) * (unsigned)K + 8 * xchunk;
            }
            const int NB = NT1 / TPB;
            auto issue_x = [&](int blk) {
                lds_byte* xs = smem + kXRing + (blk % kXSlots) * kXBlockB;
                const int kt = TPB * blk + rot1 < NT1 ? TPB * blk + rot1 : TPB * blk + rot1 - NT1;
#pragma unroll
                for (int q = 0; q < kXLoads; ++q) load_to_lds(X + xoff[q] + kt * BK, xs + q * 1024);
            };
            auto wait_blocks = [&](int n) {      // at most n blocks (kXLoads loads each) outstanding
                if (n >= 4) wait_vm<(4 * kXLoads < 64 ? 4 * kXLoads : 63)>();
                else if (n == 3) wait_vm<3 * kXLoads>();
                else if (n == 2) wait_vm<2 * kXLoads>();
                else if (n == 1) wait_vm<kXLoads>();
                else wait_vm<0>();
            };
            for (int blk = 0; blk < min(kXLead, NB); ++blk) issue_x(blk);
            wait_blocks(min(kXLead, NB) - 1);            // block 0 has landed
            __builtin_amdgcn_s_barrier();
            for (int t = 0; t < NT1; ++t) {
                const int blk = t / TPB + kXLead;
                if (t % TPB == 0 && blk < NB) issue_x(blk);
                // the consumers fetch from tile t + 2 during the next iteration
                wait_blocks(min(blk, NB - 1) - min((t + 2) / TPB, NB - 1));
                __builtin_amdgcn_s_barrier();
            }
            for (int t = 0; t < NT2 + 1; ++t) __builtin_amdgcn_s_barrier();    // phase 2: nothing to load
            continue;
        }
        // W tile: load j of this wave covers LDS chunks 64 (kWLoadsPerWave pw + j) .. + 63
        int wk[kWLoadsPerWave], wc[kWLoadsPerWave];
#pragma unroll
        for (int j = 0; j < kWLoadsPerWave; ++j) {
            const int ci = 64 * (kWLoadsPerWave * pw + j) + lane;
            const int k = ci / 48, pc = ci % 48;
            const int sw = ((k & 3) << 1) | ((k >> 3) & 1);
            wk[j] = k;
            wc[j] = ((((pc >> 1) ^ sw) << 1) | (pc & 1)) * 8;     // first element of the global chunk
        }
        // ---- phase 1 ----
        {
            unsigned woff[kWLoadsPerWave];
#pragma unroll
            for (int j = 0; j < kWLoadsPerWave; ++j)
                woff[j] = (unsigned)wk[j] * (unsigned)F + (RAGGED ? min(wc[j], fvalid - 8) : wc[j]);
            const bf16_t* wsrc = W1 + f0;
            auto issue = [&](int t) {
                lds_byte* st = smem + kRing1 + (t & (NST - 1)) * kWTileB;
                const int kt = t + rot1 < NT1 ? t + rot1 : t + rot1 - NT1;
                const bf16_t* w = wsrc + (long)kt * BK * F;
#pragma unroll
                for (int j = 0; j < kWLoadsPerWave; ++j)
                    load_to_lds(w + woff[j], st + (kWLoadsPerWave * pw + j) * 1024);
            };
            constexpr int PER = kWLoadsPerWave;
#pragma unroll
            for (int u = 0; u < DIST; ++u) issue(min(u, NT1 - 1));   // a surplus issue repeats the last tile into its own stage
            wait_vm<(DIST - 2) * PER>();     // tiles 0 and 1 have landed
            __builtin_amdgcn_s_barrier();
            for (int t = 0; t < NT1; ++t) {
                if (t + DIST < NT1) {
                    issue(t + DIST);
                    wait_vm<(DIST - 2) * PER>();   // everything up to tile t+2 has landed
                } else {
                    wait_vm<0>();
                }
                __builtin_amdgcn_s_barrier();
            }
        }
        // ---- phase 2 (the ring restarts behind Hs; all phase-1 stages are dead by now) ----
        {
            unsigned woff[kWLoadsPerWave];
#pragma unroll
            for (int j = 0; j < kWLoadsPerWave; ++j) woff[j] = (unsigned)wk[j] * (unsigned)K2 + wc[j];
            const bf16_t* wsrc = W2 + (long)f0 * K2;
            auto issue = [&](int t) {
                const int cb = t / (FS / BK), kt = (t + rot2) % (FS / BK);
                lds_byte* st = smem + kRing2 + (t & (NST - 1)) * kWTileB;
                if constexpr (RAGGED) {
                    const bf16_t* w = wsrc + cb * CB;
                    const int cvalid = min(CB, K2 - cb * CB);       // columns of this block that exist
#pragma unroll
                    for (int j = 0; j < kWLoadsPerWave; ++j) {
                        const unsigned row = (unsigned)min(kt * BK + wk[j], fvalid - 1);
                        load_to_lds(w + row * (unsigned)K2 + min(wc[j], cvalid - 8), st + (kWLoadsPerWave * pw + j) * 1024);
                    }
                } else {
                    const bf16_t* w = wsrc + (long)kt * BK * K2 + cb * CB;
#pragma unroll
                    for (int j = 0; j < kWLoadsPerWave; ++j)
                        load_to_lds(w + woff[j], st + (kWLoadsPerWave * pw + j) * 1024);
                }
            };
            constexpr int PER = kWLoadsPerWave;
#pragma unroll
            for (int u = 0; u < DIST; ++u) issue(u);      // NT2 >= 12
            wait_vm<(DIST - 2) * PER>();
            __builtin_amdgcn_s_barrier();    // matches the consumers' barrier after the Hs epilogue
            for (int t = 0; t < NT2; ++t) {
                if (t + DIST < NT2) {
                    issue(t + DIST);
                    wait_vm<(DIST - 2) * PER>();
                } else {
                    wait_vm<0>();
                }
                __builtin_amdgcn_s_barrier();
            }
        }
        continue;
    }

    // ================================== consumers ========================================
    const int i = lane & 31, h = lane >> 5;
    const int g = lane >> 4, s = lane & 15;
    const int wm = wave % WMG, wq = wave / WMG;    // row group; group of three 32-wide hidden / column tiles
    float* B1s = reinterpret_cast<float*>(smem_generic + kB1);
    for (int t = tid; t < FS; t += kConsumerWaves * 64) B1s[t] = (b1 && (!RAGGED || t < fvalid)) ? b1[f0 + t] : 0.0f;

    // lane offsets inside a weight tile for the three column tiles of this wave (k step 0, rows 0..3)
    const int sw = ((s >> 2) << 1) | (g >> 1);
    int woff[3];
#pragma unroll
    for (int t = 0; t < 3; ++t)
        woff[t] = (8 * (g >> 1) + (s >> 2)) * kRowB + (((6 * wq + 2 * t + (g & 1)) ^ sw) << 5) + 8 * (s & 3);

    // ------------------------------ phase 1 -------------------------------------------
    // Fragment sets ping-pong: with two k steps per tile (BK = 32) set 0 / 1 hold k step 0 / 1 of the
    // current tile and are re-filled for the next tile; with one k step per tile (BK = 16) set 0 / 1
    // hold even / odd tiles.  "Step" u below = k step u of the stream (tile u / KSTEPS, k step u % KSTEPS).
    {
        // byte offset of this lane's chunk in an X block: row (32 (MW wm + mt) + i), logical chunk
        // 2 (k step within the block) + h, chunk ^= (row >> 1) & 7
        int xbase[MW], xsw[MW];
#pragma unroll
        for (int mt = 0; mt < MW; ++mt) {
            const int xrow = 32 * (MW * wm + mt) + i;
            xbase[mt] = xrow * 128;
            xsw[mt] = (xrow >> 1) & 7;
        }
        f32x16 acc[MW][3];
#pragma unroll
        for (int mt = 0; mt < MW; ++mt)
#pragma unroll
            for (int t = 0; t < 3; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][t][r] = 0.0f;
        auto fetch = [&](Frag<MW>& fr, int step) {          // past the last tile: stale data, never used
            const int tile = step / KSTEPS, ks = step % KSTEPS;
            const lds_byte* st = smem + kRing1 + (tile & (NST - 1)) * kWTileB;
            const lds_byte* xs = smem + kXRing + ((tile / TPB) % kXSlots) * kXBlockB;
            const int chunk = 2 * (step & 3) + h;            // four k steps per 64-deep block
#pragma unroll
            for (int mt = 0; mt < MW; ++mt) fr.a[mt] = read_a_frag(xs + xbase[mt] + ((chunk ^ xsw[mt]) << 4));
#pragma unroll
            for (int t = 0; t < 3; ++t) fr.w[t] = read_w_frag(st + woff[t] + ks * 16 * kRowB);
        };
        auto mma = [&](const Frag<MW>& fr) {
#pragma unroll
            for (int mt = 0; mt < MW; ++mt)
#pragma unroll
                for (int u = 0; u < 3; ++u) acc[mt][u] = mfma32(fr.w[u], fr.a[mt], acc[mt][u]);
        };
        Frag<MW> f0r, f1r;
        __builtin_amdgcn_s_barrier();              // tiles 0 and 1 are in LDS
        fetch(f0r, 0);
        fetch(f1r, 1);
        // each fragment set is re-filled right after the matrix instructions that read it have been
        // issued: no copies, and the reads have most of a tile to land
        if constexpr (KSTEPS == 2) {
            for (int t = 0; t < NT1; ++t) {
                mma(f0r);
                __builtin_amdgcn_sched_barrier(0);
                fetch(f0r, 2 * t + 2);
                __builtin_amdgcn_sched_barrier(0);
                mma(f1r);
                __builtin_amdgcn_sched_barrier(0);
                fetch(f1r, 2 * t + 3);
                __builtin_amdgcn_s_barrier();
            }
        } else {
            // one k step per tile: tile t + 2 is only guaranteed to have landed after barrier t, so the
            // set freed in iteration t is re-filled at the start of iteration t + 1 (NT1 is even)
            for (int t = 0; t < NT1; t += 2) {
                mma(f0r);
                __builtin_amdgcn_sched_barrier(0);
                if (t > 0) fetch(f1r, t + 1);
                __builtin_amdgcn_s_barrier();
                mma(f1r);
                __builtin_amdgcn_sched_barrier(0);
                fetch(f0r, t + 2);
                __builtin_amdgcn_s_barrier();
            }
        }
        // epilogue: bias + activation, round to bf16, Hs[m][f] (f contiguous = phase-2 k).
        // acc rows = hidden units, columns = rows of X.
        bf16_t* Hs = reinterpret_cast<bf16_t*>(smem_generic);
        auto epilogue = [&](auto act_tag) {
            constexpr int ACT = decltype(act_tag)::value;
#pragma unroll
            for (int mt = 0; mt < MW; ++mt) {
                const int ml = 32 * (MW * wm + mt) + i;
#pragma unroll
                for (int t = 0; t < 3; ++t)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int fl = 96 * wq + 32 * t + 8 * q + 4 * h;
                        const float4 bv = *reinterpret_cast<const float4*>(B1s + fl);
                        const float v0 = apply_act<ACT>(acc[mt][t][4 * q + 0] + bv.x);
                        const float v1 = apply_act<ACT>(acc[mt][t][4 * q + 1] + bv.y);
                        const float v2 = apply_act<ACT>(acc[mt][t][4 * q + 2] + bv.z);
                        const float v3 = apply_act<ACT>(acc[mt][t][4 * q + 3] + bv.w);
                        *reinterpret_cast<uint2*>(Hs + ml * kHsLd + fl) =
                            (!RAGGED || fl < fvalid) ? make_uint2(pack_bf16(v0, v1), pack_bf16(v2, v3)) : make_uint2(0u, 0u);
                    }
            }
        };
        switch (act) {          // uniform
            case kGeluTanh: epilogue(std::integral_constant<int, kGeluTanh>()); break;
            case kRelu: epilogue(std::integral_constant<int, kRelu>()); break;
            case kRelu6: epilogue(std::integral_constant<int, kRelu6>()); break;
            default: epilogue(std::integral_constant<int, kNone>()); break;
        }
    }
    __syncthreads();       // Hs complete (workgroup barrier: the producers arrive with W2 tiles 0 and 1 landed)

    // ------------------------------ phase 2 -------------------------------------------
    {
        const bool full_block = m0 + BM <= M;
        const lds_byte* hs = smem + (32 * MW * wm + i) * (kHsLd * 2) + 16 * h;
        f32x16 acc[MW][3];         // rows = rows of X, columns = output columns
#pragma unroll
        for (int mt = 0; mt < MW; ++mt)
#pragma unroll
            for (int t = 0; t < 3; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][t][r] = 0.0f;
        constexpr int KT = FS / BK;      // tiles per column block
        auto fetch = [&](Frag<MW>& fr, int step) {
            const int tile = step / KSTEPS, ks = step % KSTEPS;
            const lds_byte* st = smem + kRing2 + (tile & (NST - 1)) * kWTileB;
            const int kbyte = (((tile + rot2) % KT) * BK + ks * 16) * 2;
#pragma unroll
            for (int mt = 0; mt < MW; ++mt) fr.a[mt] = read_a_frag(hs + mt * 32 * (kHsLd * 2) + kbyte);
#pragma unroll
            for (int t = 0; t < 3; ++t) fr.w[t] = read_w_frag(st + woff[t] + ks * 16 * kRowB);
        };
        auto mma = [&](const Frag<MW>& fr) {
#pragma unroll
            for (int mt = 0; mt < MW; ++mt)
#pragma unroll
                for (int u = 0; u < 3; ++u) acc[mt][u] = mfma32(fr.a[mt], fr.w[u], acc[mt][u]);
        };
        Frag<MW> f0r, f1r;
        fetch(f0r, 0);
        fetch(f1r, 1);
        for (int cb = 0; cb < NCB; ++cb) {
            if constexpr (KSTEPS == 2) {
                for (int kt = 0; kt < KT; ++kt) {
                    const int tile = cb * KT + kt;
                    mma(f0r);
                    __builtin_amdgcn_sched_barrier(0);
                    fetch(f0r, 2 * tile + 2);
                    __builtin_amdgcn_sched_barrier(0);
                    mma(f1r);
                    __builtin_amdgcn_sched_barrier(0);
                    fetch(f1r, 2 * tile + 3);
                    __builtin_amdgcn_s_barrier();
                }
            } else {
                for (int kt = 0; kt < KT; kt += 2) {          // KT is even
                    const int tile = cb * KT + kt;
                    mma(f0r);
                    __builtin_amdgcn_sched_barrier(0);
                    if (tile > 0) fetch(f1r, tile + 1);
                    __builtin_amdgcn_s_barrier();
                    mma(f1r);
                    __builtin_amdgcn_sched_barrier(0);
                    fetch(f0r, tile + 2);
                    __builtin_amdgcn_s_barrier();
                }
            }
            // this column block is complete: lane = output column, registers = rows of X
            // (32 lanes write 128 contiguous bytes of one row); 32-bit element offsets
#pragma unroll
            for (int mt = 0; mt < MW; ++mt) {
                const unsigned row0 = m0 + 32 * (MW * wm + mt) + 4 * h;
                if (nsplit != 1 && full_block && (!RAGGED || (cb + 1) * CB <= K2)) {   // uniform: the common case, plain stores
#pragma unroll
                    for (int t = 0; t < 3; ++t) {
                        const unsigned col = cb * CB + 96 * wq + 32 * t + i;
                        const unsigned base = ((unsigned)split * (unsigned)M + row0) * (unsigned)K2 + col;
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            part[base + (unsigned)(8 * (r >> 2) + (r & 3)) * (unsigned)K2] = acc[mt][t][r];
                            acc[mt][t][r] = 0.0f;
                        }
                    }
                } else {
#pragma unroll
                    for (int t = 0; t < 3; ++t) {
                        const unsigned col = cb * CB + 96 * wq + 32 * t + i;
                        const float bv = (nsplit == 1 && b2 && (!RAGGED || (int)col < K2)) ? b2[col] : 0.0f;
                        const unsigned base = ((nsplit == 1 ? 0u : (unsigned)split * (unsigned)M) + row0) * (unsigned)K2 + col;
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int dr = 8 * (r >> 2) + (r & 3);
                            if ((int)row0 + dr < M && (!RAGGED || (int)col < K2)) {
                                const unsigned idx = base + (unsigned)dr * (unsigned)K2;
                                if (nsplit == 1) Y[idx] = (bf16_t)(acc[mt][t][r] + bv);
                                else part[idx] = acc[mt][t][r];
                            }
                            acc[mt][t][r] = 0.0f;
                        }
                    }
                }
            }
        }
    }
    }   // row blocks of this workgroup
}

}  // namespace

bool fused_ffn_stream_ok(int M, int K, int F, int K2) {
    (void)M;
    return K % 64 == 0 && K >= 64 && F % 8 == 0 && K2 % 8 == 0 && F >= 8 && K2 >= 8;
}

template <int MW, int BK_, int CW, bool RAGGED>
static hipError_t launch_stream(const void* x, const void* w1, const float* b1, const void* w2, const float* b2,
                                void* y, int M, int K, int F, int K2, int act, void* workspace, hipStream_t s,
                                int blocks_per_wg) {
    typedef StreamCfg<MW, BK_, CW> C;
    auto kern = fused_ffn_stream_kernel<MW, BK_, CW, RAGGED>;
    if (hipError_t e = allow_dynamic_lds<fused_ffn_stream_kernel<MW, BK_, CW, RAGGED>>((int)(C::kSmem)); e != hipSuccess) return e;
    const int nsplit = (F + FS - 1) / FS;
    const int nrb = (M + C::BM - 1) / C::BM;
    dim3 grid(nsplit, (nrb + blocks_per_wg - 1) / blocks_per_wg);
    prof_start(2, s);
    prof_shape(2, grid.x * grid.y, C::kThreads);
    hipLaunchKernelGGL(kern, grid, dim3(C::kThreads), C::kSmem, s, (const bf16_t*)x, (const bf16_t*)w1, b1,
                       (const bf16_t*)w2, b2, (bf16_t*)y, (float*)workspace, M, K, F, K2, act);
    hipError_t e = hipGetLastError();
    if (nsplit != 1) prof_mid(2, s);
    if (e == hipSuccess && nsplit != 1) e = ffn_reduce((const float*)workspace, b2, y, (long)M * K2, K2, nsplit, s);
    prof_stop(2, s);      // the event pair brackets the whole entry point, the reduction included
    return e;
}

// variant 0: eight consumer waves with 32 x 96 wave tiles; 1: four consumer waves with 64 x 96 wave tiles
hipError_t fused_ffn_stream(const void* x, const void* w1, const float* b1, const void* w2, const float* b2,
                            void* y, int M, int K, int F, int K2, int act, void* workspace, hipStream_t s,
                            int variant) {
    if (!fused_ffn_stream_ok(M, K, F, K2)) return hipErrorInvalidValue;
    const bool ragged = F % FS != 0 || K2 % CB != 0;
    // Row blocks per workgroup.  Two (half as many workgroups, each twice as long, the other compute units
    // left to other streams) was measured: 47 us instead of 30 us alone and a slower concurrent step, since
    // what bounds a workgroup is its own compute unit's load path; one it stays.  Likewise 16-deep tiles in
    // an eight-stage ring (seven tiles, 84 KB, in flight instead of three, 72 KB): 31.4 us against 30.2 us,
    // so the stream is not waiting on latency either.
    const int bpw = 1;
    if (variant == 1) {
        if (ragged) return launch_stream<2, 32, 4, true>(x, w1, b1, w2, b2, y, M, K, F, K2, act, workspace, s, 1);
        return launch_stream<2, 32, 4, false>(x, w1, b1, w2, b2, y, M, K, F, K2, act, workspace, s, 1);
    }
    // the eight-consumer-wave instantiation spills a few registers once the ragged clamps are in; the
    // four-consumer-wave one (same speed) does not, so ragged shapes always take it
    if (ragged) return launch_stream<2, 32, 4, true>(x, w1, b1, w2, b2, y, M, K, F, K2, act, workspace, s, bpw);
    return launch_stream<1, 32, 8, false>(x, w1, b1, w2, b2, y, M, K, F, K2, act, workspace, s, bpw);
}

}  // namespace ago
