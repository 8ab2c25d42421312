// C = act(A W + bias) with the weight matrix pre-packed into matrix-instruction fragments (the layout of
// pack_weight): the un-fused operator of Fig. 3 / Fig. 4 built on the same inner step as the packed fused
// chain, so that fused and un-fused are compared on equal footing.  Weight fragments go from the L2
// straight into registers (one contiguous 1 KB load per wave and fragment, a ring of four k-steps ahead);
// only the activations A pass through LDS, in [row][k] tiles of KT k-values, double-buffered, one barrier
// per tile.
//
// A workgroup owns a BM x BN tile of C; its eight waves are RG row groups x CG column groups x KG k groups,
// every wave a 64 x 48 tile (4 x 3 tiles of v_mfma_f32_16x16x32_bf16, 12 matrix instructions per 7
// fragments).  The product is computed transposed, D[column of C][row of C] (weights as the A operand), so a
// lane holds 4 consecutive columns of one row of C.  With KG > 1 the k groups split every LDS tile's
// k-steps between them and their partial sums meet in LDS in group order (deterministic).
//   128 x 192, KG = 1 (KT = 128): wide outputs, e.g. 2048 x 768 -> 3072
//    64 x  96, KG = 4 (KT = 512): narrow outputs with a long reduction, e.g. 2048 x 3072 -> 768
#include "ago_dev.hpp"
#include "ago_launch.hpp"

namespace ago {
namespace {

typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512;
constexpr int kNT = 3, kPD = 4;

__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int BM, int BN, int RG, int KG>
struct PackedCfg {
    static constexpr int CG = BN / 48;
    static_assert(RG * CG * KG == 8, "eight waves");
    static constexpr int MT = BM / RG / 16;             // 16-row tiles per wave
    static constexpr int KT = 128 * KG;                 // k-values per LDS tile: four k-steps per k group
    static constexpr int AS = KT * 2 + 16;              // bytes per row of an A tile (16 mod 256: conflict-free 16-byte reads)
    static constexpr int kStage = BM * AS;
    static constexpr int UPT = BM * KT / 8 / kThreads;  // 16-byte units of an A tile per thread
    static constexpr int kReduce = (KG - 1) * RG * CG * MT * kNT * 1024;
    static constexpr int kSmem = (2 * kStage > kReduce ? 2 * kStage : kReduce);
};

template <int BM, int BN, int RG, int KG>
__global__ __launch_bounds__(kThreads) void gemm_packed_kernel(const bf16_t* __restrict__ A,
                                                               const unsigned char* __restrict__ Wp,
                                                               const float* __restrict__ bias, bf16_t* __restrict__ C,
                                                               int M, int K, int N, int act, int xcd_cols) {
    typedef PackedCfg<BM, BN, RG, KG> Cfg;
    constexpr int kMT = Cfg::MT;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int cg = wave % Cfg::CG, rg = (wave / Cfg::CG) % RG, kg = wave / (Cfg::CG * RG);
    // Workgroups are dealt to the 8 XCDs (one L2 each) round-robin in launch order.  With xcd_cols = XC > 0 the
    // grid is cut into XC x (8 / XC) rectangles, one per XCD, so that an L2 fetches only its rectangle's rows of A
    // and columns of W instead of one operand in full.
    int bx = blockIdx.x, by = blockIdx.y;
    if (xcd_cols > 0) {
        const int L = blockIdx.y * gridDim.x + blockIdx.x, xcd = L & 7, slot = L >> 3;
        const int sub_x = gridDim.x / xcd_cols, xcd_rows = 8 / xcd_cols, sub_y = gridDim.y / xcd_rows;
        bx = (xcd % xcd_cols) * sub_x + slot % sub_x;
        by = (xcd / xcd_cols) * sub_y + slot / sub_x;
    }
    const int m_blk = by * BM;
    const int ntiles = N / 16;
    const int ct0 = bx * (BN / 16) + cg * kNT;               // first column tile of this wave
    const int nt = K / Cfg::KT;                               // LDS tiles along k

    // ---- weight stream: local step j of tile t is k-step t * 4 KG + 4 kg + j
    const unsigned char* wbase = Wp + ((long)(4 * kg) * ntiles + ct0) * 1024 + lane * 16;
    const long wstep = (long)ntiles * 1024;                   // one k-step
    const long wtile = wstep * 4 * KG;                        // one LDS tile
    u32x4_t ring[kPD][kNT];
#pragma unroll
    for (int j = 0; j < kPD; ++j) {
#pragma unroll
        for (int n = 0; n < kNT; ++n) ring[j][n] = *reinterpret_cast<const u32x4_t*>(wbase + j * wstep + n * 1024);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- A tiles: a wave instruction covers 4 rows x 256 contiguous bytes
    const int r4 = lane >> 4;
    int a_row[Cfg::UPT], a_col[Cfg::UPT];
#pragma unroll
    for (int q = 0; q < Cfg::UPT; ++q) {
        const int ii = wave * Cfg::UPT + q;
        a_row[q] = (ii / (Cfg::KT / 128)) * 4 + r4;
        a_col[q] = (ii % (Cfg::KT / 128)) * 16 + i;
    }
    u32x4_t areg[Cfg::UPT];
    auto load_a = [&](int t) {
#pragma unroll
        for (int q = 0; q < Cfg::UPT; ++q)
            areg[q] = *reinterpret_cast<const u32x4_t*>(A + (long)min(m_blk + a_row[q], M - 1) * K + t * Cfg::KT + a_col[q] * 8);
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int q = 0; q < Cfg::UPT; ++q)
            *reinterpret_cast<u32x4_t*>(lds + buf * Cfg::kStage + a_row[q] * Cfg::AS + a_col[q] * 16) = areg[q];
    };
    load_a(0);
    store_a(0);
    // The first fragments are pinned here, landed, ahead of the loop: sunk into the loop's preheader in some
    // other order they make the compiler's wait counts inside the loop needlessly strict for good
#pragma unroll
    for (int j = 0; j < kPD; ++j)
#pragma unroll
        for (int n = 0; n < kNT; ++n) asm volatile("" : "+v"(ring[j][n]));
    lds_barrier();

    f32x4 acc[kMT][kNT];
#pragma unroll
    for (int m = 0; m < kMT; ++m)
#pragma unroll
        for (int n = 0; n < kNT; ++n) acc[m][n] = f32x4{0.f, 0.f, 0.f, 0.f};

    const unsigned char* abase = lds + (rg * (BM / RG) + i) * Cfg::AS + (4 * kg) * 64 + g * 16;
    for (int t = 0; t < nt; ++t) {
        const int tn = min(t + 1, nt - 1);                    // past the end: the last tile again, never used
        load_a(tn);
        __builtin_amdgcn_sched_barrier(0);
        const unsigned char* asrc = abase + (t & 1) * Cfg::kStage;
        const unsigned char* wnext = wbase + tn * wtile;
#pragma unroll
        for (int j = 0; j < kPD; ++j) {
            bf16x8 b[kMT];
#pragma unroll
            for (int m = 0; m < kMT; ++m) b[m] = *reinterpret_cast<const bf16x8*>(asrc + m * 16 * Cfg::AS + j * 64);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int m = 0; m < kMT; ++m)
#pragma unroll
                for (int n = 0; n < kNT; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ring[j][n]), b[m], acc[m][n], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int n = 0; n < kNT; ++n) ring[j][n] = *reinterpret_cast<const u32x4_t*>(wnext + j * wstep + n * 1024);
            __builtin_amdgcn_sched_barrier(0);
        }
        store_a((t + 1) & 1);
        lds_barrier();
    }

    // ---- k groups 1.. hand their partial sums to group 0 through LDS (the A tiles are no longer needed)
    if constexpr (KG > 1) {
        unsigned char* red = lds + ((rg * Cfg::CG + cg) * kMT * kNT) * 1024 + lane * 16;
        constexpr int kGroupBytes = RG * Cfg::CG * kMT * kNT * 1024;
        if (kg > 0) {
#pragma unroll
            for (int m = 0; m < kMT; ++m)
#pragma unroll
                for (int n = 0; n < kNT; ++n)
                    *reinterpret_cast<f32x4*>(red + (kg - 1) * kGroupBytes + (m * kNT + n) * 1024) = acc[m][n];
        }
        lds_barrier();
        if (kg > 0) return;
#pragma unroll
        for (int q = 0; q < KG - 1; ++q)
#pragma unroll
            for (int m = 0; m < kMT; ++m)
#pragma unroll
                for (int n = 0; n < kNT; ++n)
                    acc[m][n] += *reinterpret_cast<const f32x4*>(red + q * kGroupBytes + (m * kNT + n) * 1024);
    }

    // ---- bias, activation, bf16: lane = row of C, 4 consecutive columns per tile
#pragma unroll
    for (int n = 0; n < kNT; ++n) {
        const int col = (ct0 + n) * 16 + 4 * g;
        const f32x4 bv = bias ? *reinterpret_cast<const f32x4*>(bias + col) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int m = 0; m < kMT; ++m) {
            const int row = m_blk + rg * (BM / RG) + m * 16 + i;
            if (row < M) {
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = apply_act_rt(acc[m][n][r] + bv[r], act);
                *reinterpret_cast<uint2*>(C + (long)row * N + col) = make_uint2(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]));
            }
        }
    }
}

template <int BM, int BN, int RG, int KG>
hipError_t launch_packed_gemm(const void* a, const void* wp, const float* bias, void* c, int M, int K, int N, int act,
                              hipStream_t s) {
    typedef PackedCfg<BM, BN, RG, KG> Cfg;
    if (hipError_t e = allow_dynamic_lds<gemm_packed_kernel<BM, BN, RG, KG>>(Cfg::kSmem); e != hipSuccess) return e;
    dim3 grid(N / BN, (M + BM - 1) / BM);
    // 2 x 4 rectangles for the narrow tiling when the grid divides that way: in launch order every XCD would
    // fetch all of A (2048 x 3072 -> 768: 24.5 us in launch order, 20.6 us in rectangles).  The wide tiling
    // stays in launch order, an XCD owning column tiles (2048 x 768 -> 3072: 19.6 us against 23.2 us in rectangles).
    const int xcd_cols = (KG > 1 && grid.x % 2 == 0 && grid.y % 4 == 0 && grid.x * grid.y >= 64) ? 2 : 0;
    hipLaunchKernelGGL((gemm_packed_kernel<BM, BN, RG, KG>), grid, dim3(kThreads), Cfg::kSmem, s, (const bf16_t*)a,
                       (const unsigned char*)wp, bias, (bf16_t*)c, M, K, N, act, xcd_cols);
    return hipGetLastError();
}

}  // namespace

// 0: no tiling fits; 1: 128 x 192; 2: 64 x 96 with four k groups
int gemm_packed_variant(int M, int K, int N) {
    const bool wide = N % 192 == 0 && K % 128 == 0;
    const bool narrow = N % 96 == 0 && K % 512 == 0;
    const long wide_tiles = (long)((M + 127) / 128) * (N / 192);
    if (wide && (wide_tiles >= 192 || !narrow)) return 1;
    if (narrow) return 2;
    return 0;
}

// A third tiling, 128 x 192 with one row group and two k groups (every weight fragment loaded by one wave only,
// 96 accumulator registers), was measured at 21.6 us against 17.0 us for tiling 1 on 2048 x 768 -> 3072: the
// k-tiles take as long and the exchange of partial sums comes on top.
hipError_t gemm_packed(const void* a, const void* wp, const float* bias, void* c, int M, int K, int N, int act,
                       hipStream_t s) {
    switch (gemm_packed_variant(M, K, N)) {
        case 1: return launch_packed_gemm<128, 192, 2, 1>(a, wp, bias, c, M, K, N, act, s);
        case 2: return launch_packed_gemm<64, 96, 1, 4>(a, wp, bias, c, M, K, N, act, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ago
