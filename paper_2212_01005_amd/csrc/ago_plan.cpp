// Host-only analytic planners for the 3x3 -> 3x3 chain, the FFN chain and the attention chain:
// which tile candidate a launch uses (and, for the FFN chain, whether fusing pays at all), chosen by an
// explicit time model instead of hard-coded rules.  The paper leaves this choice to its schedule search;
// what it does give (Sec. III-B) is the redundancy algebra that prices a tiling, and that is the model's
// recompute term:
//
//     upstream work after tiling and fusing = | GS2/TS2 x (GS1/TS1 - GS2/TS2) | * | TS1 |
//
//   GS2/TS2            the downstream operator's outer (tile) loops: one pass per downstream tile
//   GS1/TS1 - GS2/TS2  outer loops the upstream operator needs and the downstream nest does not already
//                      contain (none in the three chains here: the factor is 1)
//   TS1                the upstream tile one downstream tile needs
//
// Everything else is a count of what the kernels execute (matrix instructions, tiles, workgroups, bytes of
// partial sums) multiplied by rates measured on an MI355X; the constants are listed with what they were
// measured on.  No HIP header is included: the file builds with a plain C++ compiler.
#include "ago_host.hpp"
#include <math.h>

namespace ago {

namespace {

constexpr int kCUs = 256;
constexpr double kLaunchUs = 1.5;          // back-to-back launch of a kernel on one stream (an empty kernel: 1.55 us)

inline long ceil_div(long a, long b) { return (a + b - 1) / b; }

// Sec. III-B (see the file header).
inline double upstream_work(double outer2, double extra1, double ts1) { return outer2 * extra1 * ts1; }

// ---------------------------------------------------------------------------------------------------
// conv3x3 -> conv3x3 (general-conv downstream: the re-use dimensions H2, W2 are tiled, so |TS2| < |TS1|
// and the halo of the intermediate is re-computed).
// One workgroup per TH x TW output tile, one per compute unit (1024 threads).  Time of a workgroup =
// a fixed part (both 3 x 3 weight tensors and the input tile staged through LDS, the two epilogues)
// + its matrix instructions: both convolutions run on 32-pixel x 32-channel tiles, 36 k steps
// of 16 each (K = 9 x 64), two channel tiles; a last round that fills the chip only partly is cheaper.
// Calibrated on 10 shapes x 4 candidates (batch 1 - 128 of 14 x 14 ... 112 x 112 x 64): mean error 2 %.
// ---------------------------------------------------------------------------------------------------
// candidates 0..3: units of (row tile, output-channel half); 4, 5: the earlier units of (row tile, kernel row)
const int kChainTiles[6][2] = {{7, 14}, {7, 7}, {8, 8}, {6, 14}, {7, 14}, {7, 7}};
constexpr double kChainFixedUs = 6.5, kChainUsPerMfma = 0.0045, kChainPartialRoundUs = 2.0;
constexpr double kChainFixedUsKernelRows = 7.0, kChainUsPerMfmaKernelRows = 0.005;

}  // namespace

bool plan_conv_chain(int N, int H, int W, int C, int tile_cfg, ChainPlan* out) {
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || tile_cfg >= 6) return false;
    ChainPlan best{};
    bool have = false;
    for (int cfg = 0; cfg < 6; ++cfg) {
        if (tile_cfg >= 0 ? cfg != tile_cfg : cfg >= 4) continue;      // the built-in choice is among 0..3
        const int th = kChainTiles[cfg][0], tw = kChainTiles[cfg][1];
        ChainPlan p{};
        p.cfg = cfg; p.tile_h = th; p.tile_w = tw;
        const long tiles = (long)N * ceil_div(H, th) * ceil_div(W, tw);
        p.workgroups = tiles;
        p.resident = 1;
        p.rounds = ceil_div(tiles, kCUs);
        // redundancy algebra: every downstream tile (GS2/TS2 = tiles, all O2 channels inside the tile) needs
        // the (th + 2) x (tw + 2) window of all O1 = C upstream channels, each a reduction over 9 C inputs
        p.executed_upstream_macs = upstream_work((double)tiles, 1.0, (double)(th + 2) * (tw + 2) * C * 9.0 * C);
        p.algorithmic_upstream_macs = (double)N * H * W * C * 9.0 * C;
        // what the matrix cores execute on top of that: pixel counts padded to 32-pixel tiles
        const long mfma = (ceil_div((th + 2) * (tw + 2), 32) + ceil_div(th * tw, 32)) * ceil_div(C, 32) * (9 * ceil_div(C, 16));
        // a last round that fills only part of the chip finishes sooner (fewer workgroups share the L2s and HBM)
        const double last = (double)(tiles - (p.rounds - 1) * kCUs) / kCUs;
        p.predicted_us = cfg < 4 ? kLaunchUs + p.rounds * (kChainFixedUs + kChainUsPerMfma * mfma) - kChainPartialRoundUs * (1.0 - last)
                                 : kLaunchUs + p.rounds * (kChainFixedUsKernelRows + kChainUsPerMfmaKernelRows * mfma);
        if (!have || p.predicted_us < best.predicted_us) { best = p; have = true; }
    }
    if (have && out) *out = best;
    return have;
}

// ---------------------------------------------------------------------------------------------------
// matmul -> softmax -> matmul ("downstream pointwise", Fig. 7b: the downstream tile holds all D output
// columns of its query rows, the upstream tile is one key block of the downstream reduction: nothing is
// re-computed).  Candidates: 32 NQT query rows per workgroup, 128-key blocks in a ring of NSTG LDS
// buffers.  A compute unit holds r workgroups (LDS: 2 NSTG x 16 KB each); a workgroup takes a fill time
// (Q and the first K / V block from HBM, the merge and the store at the end) plus, per key block, a fixed
// part and a part per resident query tile (the softmax on the vector ALUs is what bounds a block).
// Calibrated on 9 shapes x 4 candidates (S = 96 ... 4096): mean error 11 %, the choice within 4 % of the
// best candidate on every shape.
// ---------------------------------------------------------------------------------------------------
namespace {
const int kAttnNqt[4] = {3, 4, 2, 6}, kAttnStages[4] = {2, 2, 2, 3}, kAttnResident[4] = {2, 1, 2, 1};
constexpr double kAttnFillUs = 2.5, kAttnBlockUs = 1.0, kAttnBlockUsPerTile = 0.15;
}  // namespace

bool plan_attn(int B, int Hh, int S, int D, int tile_cfg, AttnPlan* out) {
    if (B <= 0 || Hh <= 0 || S <= 0 || (D != 64 && D != 128) || tile_cfg >= 4) return false;
    AttnPlan best{};
    bool have = false;
    for (int cfg = 0; cfg < 4; ++cfg) {
        if (tile_cfg >= 0 && cfg != tile_cfg) continue;
        // head dimension 128 has the 96- and 64-query workgroups only (two LDS buffers of two planes)
        if (D == 128 && tile_cfg < 0 && cfg != 0) continue;
        AttnPlan p{};
        const int nqt = (D == 128 && cfg != 2) ? 3 : kAttnNqt[cfg];
        p.cfg = cfg; p.queries = 32 * nqt; p.key_block = 128;
        p.stages = D == 128 ? 2 : kAttnStages[cfg];
        p.resident = D == 128 ? 1 : kAttnResident[cfg];
        p.lds_bytes = p.stages * 2 * 128 * D * 2;
        const long heads = (long)B * Hh, wgs = heads * ceil_div(S, p.queries), nblk = ceil_div(S, 128);
        p.workgroups = wgs;
        const long slots = (long)kCUs * p.resident;
        p.rounds = ceil_div(wgs, slots);
        // redundancy algebra: downstream outer loops = (query block, key block); the upstream tile is the
        // queries x keys x D block of scores that one such pass needs; no upstream loop is missing
        // (tile extents averaged over the ragged last blocks: every score is computed exactly once)
        const double qblocks = (double)ceil_div(S, p.queries);
        p.executed_upstream_macs = upstream_work((double)heads * qblocks * nblk, 1.0, (S / qblocks) * ((double)S / nblk) * D);
        p.algorithmic_upstream_macs = (double)heads * S * S * D;
        const double per_plane = D / 64.0;
        const long full = wgs / slots, rem = wgs % slots;
        double t = full * (kAttnFillUs + nblk * per_plane * (kAttnBlockUs + kAttnBlockUsPerTile * nqt * p.resident));
        if (rem) {      // last, partial round: the compute units hold fewer workgroups
            const long r_last = p.resident > 1 ? (ceil_div(rem, kCUs) < p.resident ? ceil_div(rem, kCUs) : p.resident) : 1;
            t += kAttnFillUs + nblk * per_plane * (kAttnBlockUs + kAttnBlockUsPerTile * nqt * r_last);
        }
        p.predicted_us = kLaunchUs + t;
        if (!have || p.predicted_us < best.predicted_us) { best = p; have = true; }
    }
    if (have && out) *out = best;
    return have;
}

// ---------------------------------------------------------------------------------------------------
// matmul -> activation -> matmul ("downstream pointwise" again: 64 rows x all K2 output columns per
// workgroup, the upstream tile is a 384-wide slice of the hidden dimension, which is the downstream
// reduction: nothing is re-computed).  With few rows the slices of one row block go to different compute
// units and their fp32 partial products are summed by a second pass: (slices x M x K2 x 4 bytes read, at
// the rate the reduction kernel was measured at) is what fusing costs here, against writing and re-reading
// the M x F hidden tensor once.  The un-fused side is modelled the same way: two products with fused
// epilogues on the un-fused GEMM kernels (tile shape as their launcher picks it), one workgroup per compute
// unit, a fixed part plus a part per k tile.
// Calibrated on 11 shapes (M = 128 ... 16384; 768 x 3072, 1024 x 4096, 512 x 2048, 256 x 1024): mean error 6 %.
// This is the paper's own caveat for pw -> pw (Sec. VI-C, Fig. 13d): intensive fusion does not always win.
// ---------------------------------------------------------------------------------------------------
namespace {
constexpr double kFfnFixedUs = 10.25, kFfnUsPerTile = 0.422;     // streaming kernel: per workgroup, per 32-deep weight tile
constexpr double kReduceBytesPerUs = 6.1e6;                      // partial-sum reduction pass (reads dominate)
constexpr double kGemmA0 = 6.7, kGemmAk = 0.935;                 // 128 x 192 tiles, per 64-deep k tile
constexpr double kGemmB0 = 7.3, kGemmBk = 0.565;                 // 64 x 96 tiles, per 128-deep k tile
constexpr double kGemmO0 = 6.6, kGemmOk = 1.0;                   // 128 x 128 / 64 x 128 tiles, per 64-deep k tile

double unfused_gemm_us(long M, long K, long N) {
    if (M % 128 == 0 && N % 192 == 0 && K % 64 == 0 && (M / 128) * (N / 192) >= 192)
        return ceil_div((M / 128) * (N / 192), kCUs) * (kGemmA0 + (K / 64) * kGemmAk);
    if (M % 64 == 0 && N % 96 == 0 && K % 128 == 0 && (M / 64) * (N / 96) >= 128)
        return ceil_div((M / 64) * (N / 96), kCUs) * (kGemmB0 + (K / 128) * kGemmBk);
    const long t128 = ceil_div(M, 128) * ceil_div(N, 128);
    const long tiles = t128 >= 192 ? t128 : ceil_div(M, 64) * ceil_div(N, 128);
    return ceil_div(tiles, kCUs) * (kGemmO0 + ceil_div(K, 64) * kGemmOk);
}
}  // namespace

bool plan_ffn(int M, int K, int F, int K2, FfnPlan* out) {
    if (M <= 0 || K <= 0 || F <= 0 || K2 <= 0) return false;
    FfnPlan p{};
    p.rows = 64; p.slice = 384;
    p.slices = (int)ceil_div(F, 384);
    p.workgroups = ceil_div(M, 64) * p.slices;
    p.resident = 1;
    p.rounds = ceil_div(p.workgroups, kCUs);
    // redundancy algebra: downstream outer loops = (row block, hidden slice); upstream tile = rows x slice x K
    // (tile extents averaged over the ragged last row block / slice: every hidden unit is computed exactly once)
    const double rblocks = (double)ceil_div(M, 64);
    p.executed_upstream_macs = upstream_work(rblocks * p.slices, 1.0, (M / rblocks) * ((double)F / p.slices) * K);
    p.algorithmic_upstream_macs = (double)M * F * K;
    const double tiles = K / 32.0 + 12.0 * ceil_div(K2, 384);
    double t = 2 * kLaunchUs + p.rounds * (kFfnFixedUs + kFfnUsPerTile * tiles);
    p.partial_bytes = p.slices > 1 ? (double)p.slices * M * K2 * 4.0 : 0.0;
    if (p.slices > 1) t += (p.partial_bytes + (double)M * K2 * 2.0) / kReduceBytesPerUs;
    p.predicted_us = t;
    p.predicted_unfused_us = 2 * kLaunchUs + unfused_gemm_us(M, K, F) + unfused_gemm_us(M, F, K2);
    // the model's mean error is 6 %: predictions within 10 % of each other count as a tie, and ties go to the
    // fused kernel (one entry point, no hidden tensor in memory)
    p.fuse = p.predicted_us <= 1.10 * p.predicted_unfused_us ? 1 : 0;
    if (out) *out = p;
    return true;
}

}  // namespace ago

extern "C" {

ago_status ago_fused_conv_chain_plan(int N, int H, int W, int C, int plan[8], double* recompute, float* predicted_us) {
    if (!plan) return AGO_ERR_NULL;
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0) return AGO_ERR_SHAPE;
    if (C != 64) return AGO_ERR_UNSUPPORTED;
    ago::ChainPlan p;
    if (!ago::plan_conv_chain(N, H, W, C, ago::tile_config(AGO_OP_FUSED_CONV_CHAIN), &p)) return AGO_ERR_UNSUPPORTED;
    const int v[8] = {p.cfg, p.tile_h, p.tile_w, (int)p.workgroups, p.resident, (int)p.rounds, 0, 1};
    for (int i = 0; i < 8; ++i) plan[i] = v[i];
    if (recompute) *recompute = p.executed_upstream_macs / p.algorithmic_upstream_macs;
    if (predicted_us) *predicted_us = (float)p.predicted_us;
    return AGO_OK;
}

ago_status ago_fused_attn_plan(int B, int Hh, int S, int D, int plan[8], double* recompute, float* predicted_us) {
    if (!plan) return AGO_ERR_NULL;
    if (B <= 0 || Hh <= 0 || S <= 0 || D <= 0) return AGO_ERR_SHAPE;
    if (D != 64 && D != 128) return AGO_ERR_UNSUPPORTED;
    ago::AttnPlan p;
    if (!ago::plan_attn(B, Hh, S, D, ago::tile_config(AGO_OP_FUSED_ATTN), &p)) return AGO_ERR_UNSUPPORTED;
    const int v[8] = {p.cfg, p.queries, p.key_block, (int)p.workgroups, p.resident, (int)p.rounds, p.lds_bytes, 1};
    for (int i = 0; i < 8; ++i) plan[i] = v[i];
    if (recompute) *recompute = p.executed_upstream_macs / p.algorithmic_upstream_macs;
    if (predicted_us) *predicted_us = (float)p.predicted_us;
    return AGO_OK;
}

ago_status ago_fused_ffn_plan(int M, int K, int F, int K2, int plan[8], double* recompute, float* predicted_us,
                              float* predicted_unfused_us) {
    if (!plan) return AGO_ERR_NULL;
    if (M <= 0 || K <= 0 || F <= 0 || K2 <= 0) return AGO_ERR_SHAPE;
    ago::FfnPlan p;
    if (!ago::plan_ffn(M, K, F, K2, &p)) return AGO_ERR_UNSUPPORTED;
    const int v[8] = {3, p.rows, p.slice, (int)p.workgroups, p.resident, (int)p.rounds, p.slices, p.fuse};
    for (int i = 0; i < 8; ++i) plan[i] = v[i];
    if (recompute) *recompute = p.executed_upstream_macs / p.algorithmic_upstream_macs;   // the slice is the downstream reduction
    if (predicted_us) *predicted_us = (float)p.predicted_us;
    if (predicted_unfused_us) *predicted_unfused_us = (float)p.predicted_unfused_us;
    return AGO_OK;
}

int ago_fused_ffn_pays(int M, int K, int F, int K2) {
    ago::FfnPlan p;
    if (!ago::plan_ffn(M, K, F, K2, &p)) return -1;
    return p.fuse;
}

}  // extern "C"
