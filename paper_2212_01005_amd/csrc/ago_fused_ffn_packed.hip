// Fused matmul -> activation -> matmul (pw -> pw, Sec. III-B: downstream pointwise keeps all its output
// channels in the tile and consumes the upstream result in slices of the reduction) on weights that were
// re-laid out once, ahead of time, into matrix-instruction fragments (pack_weight_kernel below).
//
// Why a second form of the kernel: with row-major [K][N] weights every weight tile has to be written
// into LDS and read back through the transposing read, and the LDS write rate (about 70 bytes per clock
// and compute unit) then bounds the loop at well under half the matrix cores' rate.  Packed weights go
// from the L2 straight into registers in the layout the matrix instruction wants (one contiguous 1 KB
// load per wave and fragment); LDS only carries the activations (x, then the hidden tile).
//
// Packed layout of a [K][N] bf16 matrix (K % 32 == 0, N % 16 == 0): fragment (ks, nt) = k-rows
// 32 ks .. 32 ks + 31, columns 16 nt .. 16 nt + 15, is 64 lanes x 8 elements, lane l holding
// W[32 ks + 8 (l / 16) + e][16 nt + l % 16], e = 0..7; fragments are stored [ks][nt][lane][e].
// That is the A operand of v_mfma_f32_16x16x32_bf16 (rows = output channels): the products are
// computed transposed, D[channel][row of x], so that a lane ends up with 4 consecutive channels of one
// row of x - 8 contiguous bytes of the hidden tile, 16 contiguous bytes of the fp32 partial result.
//
// Work split: workgroup (slice s of 384 hidden units, 64 rows of x), eight waves, wave w owning hidden
// units / output columns 48 w .. 48 w + 47 of the slice / column block.  Phase 1: Hs = act(x W1[:, s] + b1)
// as bf16 in LDS.  Phase 2: per column block of 384, P[s] = Hs W2[s, :] as fp32 partial sums
// (ffn_reduce adds the slices).  Every wave streams its own weight fragments through a ring of PD
// k-steps of registers: a slot is refilled, for the step PD ahead, right after the matrix instructions
// that consumed it, and the stream runs on across the phase boundaries (the first W2 fragments are
// requested before the activation is evaluated).
#include "ago_dev.hpp"
#include "ago_launch.hpp"
#include <type_traits>

namespace ago {
namespace {

constexpr int kBM = 64;          // rows of x per workgroup
constexpr int kFS = 384;         // hidden units per workgroup
constexpr int kCB = 384;         // output columns per column block
constexpr int kThreads = 512;    // eight waves
constexpr int kNT = 3;           // 16-wide tiles per wave: 8 x 3 x 16 = 384
constexpr int kMT = 4;           // 16-row tiles: 64 rows
constexpr int kHS = kFS * 2 + 16;   // bytes per row of the hidden tile in LDS

typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

// workgroup barrier that orders LDS traffic only: the weight loads in flight stay in flight
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ bf16x8 lds_frag(const unsigned char* p) {
    return *reinterpret_cast<const bf16x8*>(p);
}

// [K][N] row-major -> fragments.  A workgroup takes one k-step (32 rows) x 128 columns: the rows are read
// 16 bytes per thread (coalesced), parked in LDS, and every thread then gathers the 8 k-values of its
// lane for two fragments and writes them as 16 bytes.  Columns past N (N % 128 != 0) are skipped.
__global__ __launch_bounds__(256) void pack_weight_kernel(const bf16_t* __restrict__ w, u32x4_t* __restrict__ wp,
                                                          int K, int N) {
    constexpr int TN = 128, LD = TN + 8;                  // LDS row: 136 elements (272 bytes)
    __shared__ __attribute__((aligned(16))) uint16_t tile[32 * LD];
    const int ks = blockIdx.y, n0 = blockIdx.x * TN, tid = threadIdx.x;
    (void)K;
    // 32 rows x 16 units of 16 bytes = 512 units, two per thread
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int u = tid + 256 * q, r = u >> 4, c = u & 15;
        if (n0 + c * 8 < N)
            *reinterpret_cast<u32x4_t*>(&tile[r * LD + c * 8]) =
                *reinterpret_cast<const u32x4_t*>(w + (long)(32 * ks + r) * N + n0 + c * 8);
    }
    __syncthreads();
    // 8 fragments (16 columns each) x 64 lanes = 512 outputs, two per thread
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int o = tid + 256 * q, f = o >> 6, l = o & 63;
        const int col = f * 16 + (l & 15);
        if (n0 + col < N) {
            uint16_t e[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) e[t] = tile[(8 * (l >> 4) + t) * LD + col];
            wp[((long)ks * (N / 16) + n0 / 16 + f) * 64 + l] =
                u32x4_t{(unsigned)e[0] | ((unsigned)e[1] << 16), (unsigned)e[2] | ((unsigned)e[3] << 16),
                        (unsigned)e[4] | ((unsigned)e[5] << 16), (unsigned)e[6] | ((unsigned)e[7] << 16)};
        }
    }
}

// The stream of weight fragments a wave consumes: k-steps 0 .. nk1-1 of its three hidden tiles of W1,
// then for every column block the nk2 k-steps of the slice for its three column tiles of W2.  A load
// is (uniform base address) + (per lane and tile byte offset); the wave's tile offset inside a slice /
// column block is the same in both phases, so only the base moves.  Past the end the stream stays on
// its last step, so the consumer loops need no special last steps.
struct FragStream {
    const unsigned char* base;   // uniform: fragment (current k-step, tile 0 of the slice / column block)
    const unsigned char* w2_0;   // uniform: W2 fragment (first k-step of the slice, column tile 0)
    long step, step2, blk;       // bytes between k-steps (current phase; phase 2), between column blocks
    int k, nk, nk2;              // k-step inside the current segment, its length, length of a phase-2 segment
    int cb, ncb;                 // cb = -1 while in phase 1
};

__device__ __forceinline__ void load_frag_at(u32x4_t& dst, unsigned voff, const unsigned char* base) {
    dst = *reinterpret_cast<const u32x4_t*>(base + voff);
}

// voff1 / voff2 / voff2_last: byte offsets of this lane in the wave's three tiles (phase 1, phase 2, the last
// column block); they differ only for ragged shapes, where a tile beyond the matrix is redirected to tile 0
template <bool RAGGED>
__device__ __forceinline__ void issue_step(FragStream& s, u32x4_t (&slot)[kNT], const unsigned (&voff1)[kNT],
                                           const unsigned (&voff2)[kNT], const unsigned (&voff2_last)[kNT]) {
#pragma unroll
    for (int n = 0; n < kNT; ++n) {
        unsigned v = voff2[n];
        if (RAGGED) v = s.cb < 0 ? voff1[n] : (s.cb == s.ncb - 1 ? voff2_last[n] : voff2[n]);
        load_frag_at(slot[n], v, s.base);
    }
    if (++s.k == s.nk) {
        if (s.cb + 1 < s.ncb) {      // next segment: a column block of phase 2
            ++s.cb;
            s.k = 0; s.nk = s.nk2; s.step = s.step2;
            s.base = s.w2_0 + s.cb * s.blk;
        } else {                     // past the end: stay on the last step
            --s.k;
        }
    } else {
        s.base += s.step;
    }
}

template <int PD, bool RAGGED>
__global__ __launch_bounds__(kThreads) void fused_ffn_packed_kernel(
    const bf16_t* __restrict__ X, const unsigned char* __restrict__ W1p, const float* __restrict__ b1,
    const unsigned char* __restrict__ W2p, float* __restrict__ part, int M, int Mpad, int K, int F, int K2, int act, int xcd_cols) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, g = lane >> 4;
    // Launch order deals workgroups to the 8 XCDs round-robin, i.e. (8 slices) one slice per XCD.  With
    // xcd_cols = XC > 0 an XCD instead owns a rectangle of XC-th of the slices x (8 / XC)-th of the row blocks.
    int split = blockIdx.x, rb = blockIdx.y;
    if (xcd_cols > 0) {
        const int L = blockIdx.y * gridDim.x + blockIdx.x, xcd = L & 7, slot = L >> 3;
        const int sub_x = gridDim.x / xcd_cols, xcd_rows = 8 / xcd_cols, sub_y = gridDim.y / xcd_rows;
        split = (xcd % xcd_cols) * sub_x + slot % sub_x;
        rb = (xcd / xcd_cols) * sub_y + slot / sub_x;
    }
    const int m0 = rb * kBM;
    const int XS = K * 2 + 16;                       // bytes per row of the x tile in LDS
    const int ftiles = F / 16, ctiles = K2 / 16;
    const int nk1 = K / 32;
    const int fs = min(kFS, F - split * kFS);        // hidden units of this slice
    const int nk2 = fs / 32;
    const int ncb = (K2 + kCB - 1) / kCB;
    const int ft0 = split * (kFS / 16) + wave * kNT; // first hidden tile of this wave
    const int ct0 = wave * kNT;                      // first column tile of this wave inside a column block

    // ---- bias of this wave's hidden units: 4 consecutive units per lane and tile
    f32x4 bias1[kNT];
#pragma unroll
    for (int n = 0; n < kNT; ++n) {
        const int f = (ft0 + n) * 16 + 4 * g;
        bias1[n] = (b1 && f < F) ? *reinterpret_cast<const f32x4*>(b1 + f) : f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // ---- the weight stream, PD k-steps ahead (a fragment is 1024 bytes)
    FragStream s;
    s.base = W1p + (long)split * (kFS / 16) * 1024;
    s.w2_0 = W2p + (long)split * (kFS / 32) * ctiles * 1024;
    s.step = (long)ftiles * 1024;
    s.step2 = (long)ctiles * 1024;
    s.blk = (long)(kCB / 16) * 1024;
    s.k = 0; s.nk = nk1; s.nk2 = nk2; s.cb = -1; s.ncb = ncb;
    unsigned voff1[kNT], voff2[kNT], voff2_last[kNT];
#pragma unroll
    for (int n = 0; n < kNT; ++n) {
        voff2[n] = (unsigned)((ct0 + n) * 1024 + lane * 16);
        voff1[n] = (RAGGED && ft0 + n >= ftiles) ? (unsigned)(lane * 16) : voff2[n];
        voff2_last[n] = (RAGGED && (ncb - 1) * (kCB / 16) + ct0 + n >= ctiles) ? (unsigned)(lane * 16) : voff2[n];
    }
    u32x4_t ring[PD][kNT];
#pragma unroll
    for (int j = 0; j < PD; ++j) {
        issue_step<RAGGED>(s, ring[j], voff1, voff2, voff2_last);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- x tile -> LDS (rows beyond M repeat the last row; their results are never read).  A wave
    // instruction covers 4 rows x 256 contiguous bytes (16 lanes x 16 bytes: every LDS bank once per row);
    // wave w stages rows 8 w .. 8 w + 7; up to 16 loads in flight per lane
    {
        const int upr = K / 8;                       // 16-byte units per row
        const int r4 = lane >> 4;
        for (int c0 = 0; c0 < upr; c0 += 128) {
            u32x4_t v[16];
#pragma unroll
            for (int t = 0; t < 16; ++t) {
                const int c = min(c0 + 16 * (t >> 1) + i, upr - 1);
                const int r = 8 * wave + 4 * (t & 1) + r4;
                v[t] = *reinterpret_cast<const u32x4_t*>(X + (long)min(m0 + r, M - 1) * K + c * 8);
            }
#pragma unroll
            for (int t = 0; t < 16; ++t) {
                const int c = min(c0 + 16 * (t >> 1) + i, upr - 1);
                const int r = 8 * wave + 4 * (t & 1) + r4;
                *reinterpret_cast<u32x4_t*>(lds + r * XS + c * 16) = v[t];
            }
        }
    }
    __syncthreads();      // also drains the first fragments: nothing to overlap with yet

    f32x4 acc[kMT][kNT];
#pragma unroll
    for (int m = 0; m < kMT; ++m)
#pragma unroll
        for (int n = 0; n < kNT; ++n) acc[m][n] = f32x4{0.f, 0.f, 0.f, 0.f};

    // one k-step: 12 matrix instructions on the slot's weight fragments and the activation fragments `cur`
    // (read from LDS during the previous step), the next step's activation fragments requested into `nxt` ahead
    // of them, the slot refilled PD steps ahead after them.  The scheduling barriers keep the order as written:
    // left to itself the compiler sinks the loads down to their use and nothing runs ahead any more.
    auto step = [&](u32x4_t (&slot)[kNT], const bf16x8 (&cur)[kMT], bf16x8 (&nxt)[kMT], const unsigned char* next_src,
                    int row_stride) {
#pragma unroll
        for (int m = 0; m < kMT; ++m) nxt[m] = lds_frag(next_src + m * 16 * row_stride);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < kMT; ++m)
#pragma unroll
            for (int n = 0; n < kNT; ++n)
                acc[m][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, slot[n]), cur[m], acc[m][n], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        issue_step<RAGGED>(s, slot, voff1, voff2, voff2_last);
        __builtin_amdgcn_sched_barrier(0);
    };
    // a loop of nk k-steps (a multiple of PD, PD even) over activation rows at `src`; the fragments of the step
    // after the last are read from the last step's address again and dropped
    bf16x8 frag[2][kMT];
    auto k_loop = [&](const unsigned char* src, int row_stride, int nk) {
#pragma unroll
        for (int m = 0; m < kMT; ++m) frag[0][m] = lds_frag(src + m * 16 * row_stride);
        for (int k = 0; k < nk; k += PD) {
#pragma unroll
            for (int j = 0; j < PD; ++j)
                step(ring[j], frag[j & 1], frag[(j + 1) & 1], src + min(k + j + 1, nk - 1) * 64, row_stride);
        }
    };

    // ---- phase 1: D[hidden unit][row of x] += W1 fragment x x fragment
    k_loop(lds + i * XS + g * 16, XS, nk1);
    lds_barrier();        // every wave is done reading x: the hidden tile takes its place

    // ---- activation, bf16, into LDS as [row of x][hidden unit of the slice]
    auto hidden_to_lds = [&](auto actc) {
        constexpr int ACT = decltype(actc)::value;
#pragma unroll
        for (int m = 0; m < kMT; ++m)
#pragma unroll
            for (int n = 0; n < kNT; ++n) {
                float h[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) h[r] = apply_act<ACT>(acc[m][n][r] + bias1[n][r]);
                *reinterpret_cast<uint2*>(lds + (m * 16 + i) * kHS + (wave * 48 + n * 16 + 4 * g) * 2) =
                    make_uint2(pack_bf16(h[0], h[1]), pack_bf16(h[2], h[3]));
                acc[m][n] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
    };
    switch (act) {
        case kGeluTanh: hidden_to_lds(std::integral_constant<int, kGeluTanh>{}); break;
        case kRelu: hidden_to_lds(std::integral_constant<int, kRelu>{}); break;
        case kRelu6: hidden_to_lds(std::integral_constant<int, kRelu6>{}); break;
        default: hidden_to_lds(std::integral_constant<int, kNone>{}); break;
    }
    lds_barrier();

    // ---- phase 2: per column block, D[output column][row of x] += W2 fragment x hidden fragment
    const unsigned char* hb = lds + i * kHS + g * 16;
    for (int cb = 0; cb < ncb; ++cb) {
        k_loop(hb, kHS, nk2);
        // partial sums of this block: lane = row of x, 4 consecutive output columns per tile
#pragma unroll
        for (int n = 0; n < kNT; ++n) {
            const int ct = cb * (kCB / 16) + ct0 + n;
            if (!RAGGED || ct < ctiles) {
#pragma unroll
                for (int m = 0; m < kMT; ++m) {
                    float* dst = part + ((long)split * Mpad + m0 + m * 16 + i) * K2 + ct * 16 + 4 * g;
                    *reinterpret_cast<f32x4*>(dst) = acc[m][n];
                }
            }
#pragma unroll
            for (int m = 0; m < kMT; ++m) acc[m][n] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }
    // the loads still in flight target registers only; the wave ends once they have landed
}

}  // namespace

bool fused_ffn_packed_ok(int M, int K, int F, int K2) {
    (void)M;
    // x tile or hidden tile in LDS; k-steps of x and of every hidden slice in pairs; whole fragments
    return K % 64 == 0 && K >= 64 && F % 64 == 0 && F >= 64 && K2 % 16 == 0 && K2 >= 16 &&
           (long)kBM * (K * 2 + 16) <= 160 * 1024;
}

long fused_ffn_packed_rows(int M) { return ((long)M + kBM - 1) / kBM * kBM; }
int fused_ffn_packed_nsplit(int F) { return (F + kFS - 1) / kFS; }

hipError_t pack_weight(const void* w, void* wp, int K, int N, hipStream_t s) {
    dim3 grid((N + 127) / 128, K / 32);
    hipLaunchKernelGGL(pack_weight_kernel, grid, dim3(256), 0, s, (const bf16_t*)w, (u32x4_t*)wp, K, N);
    return hipGetLastError();
}

template <int PD, bool RAGGED>
static hipError_t launch_packed(const void* x, const void* w1p, const float* b1, const void* w2p, const float* b2,
                                void* y, int M, int K, int F, int K2, int act, void* workspace, hipStream_t s) {
    const int lds_bytes = kBM * max(K * 2 + 16, kHS);
    if (hipError_t e = allow_dynamic_lds<fused_ffn_packed_kernel<PD, RAGGED>>(lds_bytes); e != hipSuccess) return e;
    const int nsplit = fused_ffn_packed_nsplit(F);
    const long Mpad = fused_ffn_packed_rows(M);
    dim3 grid(nsplit, (unsigned)(Mpad / kBM));
    // An XCD (one L2) per slice, which launch order gives with 8 slices, makes every XCD fetch all of x at the
    // start of the kernel; rectangles of half the slices x a quarter of the row blocks cut that burst to a
    // quarter (x in LDS after 3.7 us instead of 5.3 us at 2048 rows) at the price of four XCDs streaming each
    // slice's weights, which spreads over the whole kernel.
    const int xcd_cols = (grid.x % 2 == 0 && grid.y % 4 == 0) ? 2 : 0;
    prof_start(2, s);
    prof_shape(2, grid.x * grid.y, kThreads);
    hipLaunchKernelGGL((fused_ffn_packed_kernel<PD, RAGGED>), grid, dim3(kThreads), lds_bytes, s, (const bf16_t*)x,
                       (const unsigned char*)w1p, b1, (const unsigned char*)w2p, (float*)workspace, M, (int)Mpad, K, F, K2, act, xcd_cols);
    hipError_t e = hipGetLastError();
    prof_mid(2, s);
    if (e == hipSuccess) e = ffn_reduce((const float*)workspace, b2, y, (long)M * K2, K2, nsplit, s, Mpad * K2);
    prof_stop(2, s);
    return e;
}

hipError_t fused_ffn_packed(const void* x, const void* w1p, const float* b1, const void* w2p, const float* b2,
                            void* y, int M, int K, int F, int K2, int act, void* workspace, hipStream_t s) {
    if (!fused_ffn_packed_ok(M, K, F, K2)) return hipErrorInvalidValue;
    const bool ragged = F % kFS != 0 || K2 % kCB != 0;
    const bool deep = K % 128 == 0 && F % 128 == 0 && (F % kFS) % 128 == 0;   // k-steps in fours everywhere
    if (deep) {
        if (ragged) return launch_packed<4, true>(x, w1p, b1, w2p, b2, y, M, K, F, K2, act, workspace, s);
        return launch_packed<4, false>(x, w1p, b1, w2p, b2, y, M, K, F, K2, act, workspace, s);
    }
    if (ragged) return launch_packed<2, true>(x, w1p, b1, w2p, b2, y, M, K, F, K2, act, workspace, s);
    return launch_packed<2, false>(x, w1p, b1, w2p, b2, y, M, K, F, K2, act, workspace, s);
}

}  // namespace ago
