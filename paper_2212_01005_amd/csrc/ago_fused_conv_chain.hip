// Fused conv3x3 -> conv3x3, 64 -> 64 -> 64 channels, bf16 (AGO Sec. III-B, Fig. 5: a general
// convolution downstream re-uses the upstream result on O2, H2 and W2, so spatial tiling of the
// downstream operator costs recomputation of a one-pixel halo of the upstream operator:
// executed upstream work = ((TH+2)(TW+2)) / (TH TW) of the un-fused count).
//
// One workgroup owns a TH x TW tile of output pixels of one image:
//   load   X tile with a 2-pixel halo, (TH+4) x (TW+4) x 64, zero outside the image -> LDS
//          all nine taps of Wa, transposed to [tap][out][in] -> LDS (83 KB)
//   conv1  T = relu(conv3x3(X) + ba) on the (TH+2) x (TW+2) region -> LDS (bf16), T := 0 outside
//          the image (the intermediate is what the second convolution pads).  No barrier inside:
//          everything conv1 reads is resident.  Meanwhile Wb is prefetched into registers.
//   swap   barrier, Wb registers -> the weight area of LDS, barrier
//   conv2  Y = relu(conv3x3(T) + bb (+ X)) on TH x TW -> global memory
// Both convolutions are implicit GEMMs [pixels] x [9 taps x 64] x [64] on 32x32x16 bf16 matrix
// instructions.  The work of each convolution is dealt out as (32-pixel row tile, half of the output
// channels) units, one per wave, each running all nine taps over all 64 input channels into one accumulator:
// 10 units for conv1 and 8 for conv2 at 7 x 14, two to three waves per SIMD, and nothing to exchange afterwards.
// (The earlier cut, (row tile, kernel row) units whose three partial sums met in LDS, needed one activation
// fragment per two matrix instructions instead of one per one, but paid 2.8 us for the two exchanges; it is
// kept as tile configurations 4 and 5: 12.5 us against 10.9 us on 8 x 56 x 56 x 64.)
//
// LDS layouts.  A 16-byte-per-lane fragment read is served one half-wave (32 lanes) at a time and is
// bank-conflict free when the 32 rows it touches are 144 bytes apart (72-element rows) or fall into
// two runs of 16 such rows whose starts differ by a multiple of 256 bytes (measured with the LDS
// bank-conflict counter).  Weights: row = output channel, 8 chunks of 8 input channels, 72-element
// rows, chunk index XOR-ed with (row >> 5) & 1 (constant within a fragment read; it only spreads the
// transposing stores).  Activation tiles: 72 elements per pixel, pixel rows padded to a multiple of
// 256 bytes, and every half-wave of a fragment read covers 16 consecutive pixels of two tile rows.
#include "ago_dev.hpp"
#include "ago_launch.hpp"
#include "ago_host.hpp"

namespace ago {

template <int TH, int TW>
struct ChainGeom {
    static constexpr int C = 64, LD = C + 8;
    static constexpr int XH = TH + 4, XW = TW + 4, R1H = TH + 2, R1W = TW + 2;
    // A 16-byte fragment read is conflict-free when the two pixel rows that the 32 lanes of a
    // half-wave cover start a multiple of 256 bytes apart: rows of the X and T tiles are padded
    // to that pitch (elements).
    static constexpr int XROW = (XW * LD * 2 + 255) / 256 * 128, TROW = (R1W * LD * 2 + 255) / 256 * 128;
    // conv2 lays its output pixels out 16 to a lane row when the tile is 9..16 wide (so that a
    // half-wave covers exactly two rows of T); narrower tiles keep the dense numbering
    static constexpr int P2W = (TW > 8 && TW <= 16) ? 16 : TW;
    static constexpr int P1 = R1H * R1W, P2 = TH * P2W;
    static constexpr int NMT1 = (P1 + 31) / 32, NMT2 = (P2 + 31) / 32;
    static constexpr size_t kSmem = ((size_t)XH * XROW + R1H * TROW + 9 * 64 * LD) * 2 + 128 * 4;
};

// One convolution over an LDS-resident source tile.  The work is cut into units of (32-pixel row
// tile, kernel row): 3 NMT of them, one per wave (the remaining waves idle).  A unit runs the three
// taps of its kernel row over all 64 input channels for both 32-channel halves of the output, so
// every activation fragment feeds two matrix instructions (two independent accumulators); the three
// partial sums of a row tile are added through LDS, each unit reducing and finishing a third of
// the tile's channels.
// SRC_ROW = elements per pixel row of the source tile, DST_P = lanes per destination row (pixel
// m sits at row m / DST_P, column m % DST_P; columns >= DST_W are padding), NP = destination
// lane slots, NMT = row tiles.  Weights are MFMA operand A: accumulator rows = output channels,
// columns = pixels.
template <int SRC_ROW, int DST_P, int DST_W, int NP, int NMT>
struct ConvStage {
    static constexpr int LD = 72;
    static constexpr int NU = 3 * NMT;                  // units
    static_assert(NU <= 16, "one unit per wave");
    f32x16 acc[2];                                      // output channels 0..31, 32..63
    int off;                                            // LDS offset of this lane's pixel, kernel row tg, column 0
    int wbase;                                          // LDS offset of this lane's weight row, kernel row tg

    __device__ __forceinline__ static bool live(int wave) { return wave < NU; }
    __device__ __forceinline__ static int tile(int wave) { return wave / 3; }
    __device__ __forceinline__ static int tg(int wave) { return wave % 3; }

    __device__ __forceinline__ void init(int wave, int j, int h) {
        int m = tile(wave) * 32 + j;
        if (m >= NP) m = 0;
        const int px = (m % DST_P) < DST_W ? m % DST_P : 0;      // padding lanes read a valid pixel
        off = (m / DST_P + tg(wave)) * SRC_ROW + px * LD + 8 * h;
        wbase = (tg(wave) * 3 * 64 + j) * LD;
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc[0][r] = 0.f; acc[1][r] = 0.f; }
    }

    struct Frag { bf16x8 x, w0, w1; };
    // step = (kernel column) * 4 + k step; the weight rows of output channels 32..63 carry the
    // chunk swizzle bit (row >> 5)
    __device__ __forceinline__ Frag fetch(const bf16_t* src, const bf16_t* ws, int step, int h) const {
        const int col = step >> 2, ks = step & 3;
        Frag f;
        f.x = ld_bf16x8(src + off + col * LD + ks * 16);
        f.w0 = ld_bf16x8(ws + wbase + col * 64 * LD + ((ks * 2 + h) << 3));
        f.w1 = ld_bf16x8(ws + wbase + (col * 64 + 32) * LD + (((ks * 2 + h) ^ 1) << 3));
        return f;
    }

    // 3 taps x 4 k-steps, fully unrolled, with the LDS fragment reads issued DEPTH steps ahead of
    // the matrix instructions that consume them.  src = activation tile, ws = [9][64][LD] weights.
    __device__ __forceinline__ void run(const bf16_t* src, const bf16_t* ws, int h) {
        constexpr int DEPTH = 3, STEPS = 12;
        Frag q[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) q[d] = fetch(src, ws, d, h);
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const Frag cur = q[s % DEPTH];
            if (s + DEPTH < STEPS) q[s % DEPTH] = fetch(src, ws, s + DEPTH, h);
            acc[0] = mfma32(cur.w0, cur.x, acc[0]);
            acc[1] = mfma32(cur.w1, cur.x, acc[1]);
        }
    }

    // Sum the three kernel-row partial accumulators of every row tile.  The accumulators are cut
    // into 8 groups of 4 registers (group = channel half * 4 + g: output channels 32 n + 8 g + 4 h
    // .. + 3 of this lane's pixel); the unit of kernel row 0 owns groups 0..2, row 1 groups 3..5,
    // row 2 groups 6, 7.  Every unit parks the groups it does not own in `scratch`
    // ([tile][group][source slot 0 / 1][64 lanes] float4, 16 KB per tile) and, after a barrier,
    // adds the two parked copies of the groups it owns, so that the reduction and the epilogue
    // are spread over all units.  The caller places barriers before (scratch no longer read as
    // weights) and between the two halves.
    __device__ __forceinline__ static int owner_of(int grp) { return grp < 3 ? 0 : grp < 6 ? 1 : 2; }
    __device__ __forceinline__ void park(float* scratch, int wave, int lane) const {
        const int me = tg(wave);
        float4* base = reinterpret_cast<float4*>(scratch) + tile(wave) * 16 * 64 + lane;
#pragma unroll
        for (int grp = 0; grp < 8; ++grp) {
            const int ow = grp < 3 ? 0 : grp < 6 ? 1 : 2;
            if (me == ow) continue;
            // the two sources of a group are the non-owners in increasing order
            const int slot = me > ow ? me - 1 : me;
            const int n = grp >> 2, g = grp & 3;
            base[(grp * 2 + slot) * 64] = make_float4(acc[n][4 * g], acc[n][4 * g + 1], acc[n][4 * g + 2], acc[n][4 * g + 3]);
        }
    }
    // adds the parked copies into the owned groups (the other groups of acc are left as they are)
    __device__ __forceinline__ void gather(const float* scratch, int wave, int lane) {
        const int me = tg(wave);
        const float4* base = reinterpret_cast<const float4*>(scratch) + tile(wave) * 16 * 64 + lane;
#pragma unroll
        for (int grp = 0; grp < 8; ++grp) {
            const int ow = grp < 3 ? 0 : grp < 6 ? 1 : 2;
            if (me != ow) continue;
            const int n = grp >> 2, g = grp & 3;
            const float4 u = base[(grp * 2) * 64], v = base[(grp * 2 + 1) * 64];
            acc[n][4 * g] += u.x + v.x; acc[n][4 * g + 1] += u.y + v.y;
            acc[n][4 * g + 2] += u.z + v.z; acc[n][4 * g + 3] += u.w + v.w;
        }
    }
};

// The other way to cut a convolution into units: (32-pixel row tile, half of the output channels), 2 NMT of
// them, each running all nine taps.  One accumulator per unit and nothing to exchange afterwards, at the
// price of one activation fragment per matrix instruction instead of one per two.
template <int SRC_ROW, int DST_P, int DST_W, int NP, int NMT>
struct ConvStageFull {
    static constexpr int LD = 72;
    static constexpr int NU = 2 * NMT;
    static_assert(NU <= 16, "one unit per wave");
    f32x16 acc;                                         // output channels 32 half .. 32 half + 31
    int off;                                            // LDS offset of this lane's pixel, kernel row 0, column 0
    int wbase;                                          // LDS offset of this lane's weight row, tap 0
    int swz;

    __device__ __forceinline__ static bool live(int wave) { return wave < NU; }
    __device__ __forceinline__ static int tile(int wave) { return wave >> 1; }
    __device__ __forceinline__ static int half(int wave) { return wave & 1; }

    __device__ __forceinline__ void init(int wave, int j, int h) {
        int m = tile(wave) * 32 + j;
        if (m >= NP) m = 0;
        const int px = (m % DST_P) < DST_W ? m % DST_P : 0;
        off = (m / DST_P) * SRC_ROW + px * LD + 8 * h;
        wbase = (half(wave) * 32 + j) * LD;
        swz = half(wave);
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    }
    struct Frag { bf16x8 x, w; };
    __device__ __forceinline__ Frag fetch(const bf16_t* src, const bf16_t* ws, int step, int h) const {
        const int tap = step >> 2, ks = step & 3, kr = tap / 3, col = tap % 3;
        Frag f;
        f.x = ld_bf16x8(src + off + kr * SRC_ROW + col * LD + ks * 16);
        f.w = ld_bf16x8(ws + wbase + tap * 64 * LD + (((ks * 2 + h) ^ swz) << 3));
        return f;
    }
    __device__ __forceinline__ void run(const bf16_t* src, const bf16_t* ws, int h) {
        constexpr int DEPTH = 4, STEPS = 36;
        Frag q[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) q[d] = fetch(src, ws, d, h);
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const Frag cur = q[s % DEPTH];
            if (s + DEPTH < STEPS) q[s % DEPTH] = fetch(src, ws, s + DEPTH, h);
            acc = mfma32(cur.w, cur.x, acc);
        }
    }
};

// All nine taps of one weight tensor [3][3][64 in][64 out] -> LDS [tap][out][in]: 9 * 128 transposition
// units of [8 in][4 out]; unit u -> tap u / 128, out-channel quad (u & 15), in-channel octet (u >> 4) & 7.
__device__ __forceinline__ void load_weight_unit(const bf16_t* Wsrc, int u, uint2 (&r)[8]) {
    constexpr int C = 64;
    const int tap = u >> 7, nq = u & 15, ko = (u >> 4) & 7;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
        r[kk] = *reinterpret_cast<const uint2*>(Wsrc + ((long)tap * C + ko * 8 + kk) * C + nq * 4);
}
__device__ __forceinline__ void store_weight_unit(bf16_t* Ws, int u, const uint2 (&r)[8]) {
    constexpr int LD = 72;
    const int tap = u >> 7, nq = u & 15, ko = (u >> 4) & 7;
    // Transpose the [8 in][4 out] block one output channel at a time.  In store t lane nq writes
    // output channel 4 nq + ((t + nq + nq / 4) & 3): with that rotation (and the row >> 5 swizzle)
    // the 16-byte stores of a wave, whose rows are 4 apart, are bank-conflict free.
    const int rot = nq + (nq >> 2);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int q = (t + rot) & 3;
        const bool hi_word = q & 2;
        const int sh = (q & 1) << 4;
        uint32_t v[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const uint32_t e = hi_word ? r[2 * m].y : r[2 * m].x;
            const uint32_t d = hi_word ? r[2 * m + 1].y : r[2 * m + 1].x;
            v[m] = ((e >> sh) & 0xffffu) | ((d >> sh) << 16);
        }
        const int o = nq * 4 + q;
        st_u4(Ws + (tap * 64 + o) * LD + ((ko ^ ((o >> 5) & 1)) << 3), make_uint4(v[0], v[1], v[2], v[3]));
    }
}

template <int TH, int TW, bool FULL = true>
__global__ __launch_bounds__(1024) void fused_conv_chain_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ Wa, const float* __restrict__ ba,
    const bf16_t* __restrict__ Wb, const float* __restrict__ bb, bf16_t* __restrict__ Y,
    int H, int W, int tiles_h, int tiles_w, int residual) {
    typedef ChainGeom<TH, TW> G;
    constexpr int C = G::C, LD = G::LD, XW = G::XW, R1W = G::R1W, P1 = G::P1, P2 = G::P2;
    constexpr int XROW = G::XROW, TROW = G::TROW, P2W = G::P2W;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* Xs = reinterpret_cast<bf16_t*>(smem);      // [XH][XROW]: pixel (r, x) at r * XROW + x * LD
    bf16_t* Ts = Xs + G::XH * XROW;                    // [R1H][TROW]
    bf16_t* Ws = Ts + G::R1H * TROW;                   // [9][64][LD]  (tap, out channel, in channel)
    float* Bias = reinterpret_cast<float*>(Ws + 9 * 64 * LD);   // ba[64], bb[64] (0 when absent)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 31, h = lane >> 5;
    int b = blockIdx.x;
    const int tw = b % tiles_w; b /= tiles_w;
    const int th = b % tiles_h;
    const int n = b / tiles_h;
    const int oh0 = th * TH, ow0 = tw * TW;
    X += (long)n * H * W * C;
    Y += (long)n * H * W * C;

    // Wa / Wb: unit u < 1024 belongs to thread u and may stay in registers for a long time (the second weight
    // tensor is prefetched during conv1); the remaining 128 units are loaded and stored in one go by the
    // first 128 threads, so that only 16 registers are held across conv1.
    uint2 rw[8];
    auto load_w = [&](const bf16_t* Wsrc) { load_weight_unit(Wsrc, tid, rw); };
    auto store_w = [&](const bf16_t* Wsrc) {
        uint2 extra[8];
        if (tid < 9 * 128 - 1024) load_weight_unit(Wsrc, 1024 + tid, extra);
        store_weight_unit(Ws, tid, rw);
        if (tid < 9 * 128 - 1024) store_weight_unit(Ws, 1024 + tid, extra);
    };

    load_w(Wa);
    if (tid < 128) Bias[tid] = tid < 64 ? (ba ? ba[tid] : 0.0f) : (bb ? bb[tid - 64] : 0.0f);
    for (int it = tid; it < G::XH * XW * 8; it += 1024) {
        const int pix = it >> 3, kc = it & 7;
        const int ih = oh0 - 2 + pix / XW, iw = ow0 - 2 + pix % XW;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (ih >= 0 && ih < H && iw >= 0 && iw < W) v = ld_u4(X + ((long)ih * W + iw) * C + kc * 8);
        st_u4(Xs + (pix / XW) * XROW + (pix % XW) * LD + kc * 8, v);
    }
    store_w(Wa);
    __syncthreads();
    load_w(Wb);            // in flight during conv1

    // ---- conv1: rows = output channels (weights are operand A), cols = region pixels --------
    if constexpr (FULL) {
        typedef ConvStageFull<XROW, R1W, R1W, P1, G::NMT1> Stage;
        Stage st;
        if (Stage::live(wave)) {
            st.init(wave, j, h);
            st.run(Xs, Ws, h);
            const int m = Stage::tile(wave) * 32 + j;
            if (m < P1) {
                const int y = oh0 - 1 + m / R1W, x = ow0 - 1 + m % R1W;
                const bool inside = y >= 0 && y < H && x >= 0 && x < W;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int o = Stage::half(wave) * 32 + 8 * g + 4 * h;
                    uint2 v = make_uint2(0, 0);
                    if (inside) {
                        const float4 bv = *reinterpret_cast<const float4*>(Bias + o);
                        v = make_uint2(pack_bf16(fmaxf(st.acc[4 * g] + bv.x, 0.f), fmaxf(st.acc[4 * g + 1] + bv.y, 0.f)),
                                       pack_bf16(fmaxf(st.acc[4 * g + 2] + bv.z, 0.f), fmaxf(st.acc[4 * g + 3] + bv.w, 0.f)));
                    }
                    *reinterpret_cast<uint2*>(Ts + (m / R1W) * TROW + (m % R1W) * LD + o) = v;
                }
            }
        }
    } else {
        typedef ConvStage<XROW, R1W, R1W, P1, G::NMT1> Stage;
        Stage st;
        const bool live = Stage::live(wave);
        const int me = Stage::tg(wave);
        if (live) {
            st.init(wave, j, h);
            st.run(Xs, Ws, h);
        }
        __syncthreads();                       // Wa is dead: its LDS area becomes reduction scratch
        if (live) st.park(reinterpret_cast<float*>(Ws), wave, lane);
        __syncthreads();
        if (live) {
            st.gather(reinterpret_cast<const float*>(Ws), wave, lane);
            // epilogue of the owned groups: bias + ReLU, zero outside the image, bf16 -> Ts[pixel][channel]
            const int m = Stage::tile(wave) * 32 + j;
            if (m < P1) {
                const int y = oh0 - 1 + m / R1W, x = ow0 - 1 + m % R1W;
                const bool inside = y >= 0 && y < H && x >= 0 && x < W;
#pragma unroll
                for (int grp = 0; grp < 8; ++grp) {
                    if (Stage::owner_of(grp) != me) continue;
                    const int ot = grp >> 2, g = grp & 3;
                    const int o = ot * 32 + 8 * g + 4 * h;
                    uint2 v = make_uint2(0, 0);
                    if (inside) {
                        const float4 bv = *reinterpret_cast<const float4*>(Bias + o);
                        v = make_uint2(pack_bf16(fmaxf(st.acc[ot][4 * g] + bv.x, 0.f), fmaxf(st.acc[ot][4 * g + 1] + bv.y, 0.f)),
                                       pack_bf16(fmaxf(st.acc[ot][4 * g + 2] + bv.z, 0.f), fmaxf(st.acc[ot][4 * g + 3] + bv.w, 0.f)));
                    }
                    *reinterpret_cast<uint2*>(Ts + (m / R1W) * TROW + (m % R1W) * LD + o) = v;
                }
            }
        }
    }
    __syncthreads();       // Ts complete, reduction scratch no longer read
    store_w(Wb);           // Wb -> LDS
    __syncthreads();

    // ---- conv2: rows = output channels, cols = output pixels --------------------------------
    if constexpr (FULL) {
        typedef ConvStageFull<TROW, P2W, TW, P2, G::NMT2> Stage;
        Stage st;
        if (Stage::live(wave)) {
            st.init(wave, j, h);
            st.run(Ts, Ws, h);
            const int m = Stage::tile(wave) * 32 + j;
            const int py = m / P2W, px = m % P2W;
            const int y = oh0 + py, x = ow0 + px;
            if (m < P2 && px < TW && y < H && x < W) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int o = Stage::half(wave) * 32 + 8 * g + 4 * h;
                    float4 v = make_float4(st.acc[4 * g], st.acc[4 * g + 1], st.acc[4 * g + 2], st.acc[4 * g + 3]);
                    const float4 bv = *reinterpret_cast<const float4*>(Bias + 64 + o);
                    v.x += bv.x; v.y += bv.y; v.z += bv.z; v.w += bv.w;
                    if (residual) {
                        const uint2 xr = *reinterpret_cast<const uint2*>(Xs + (py + 2) * XROW + (px + 2) * LD + o);
                        v.x += lo_bf16(xr.x); v.y += hi_bf16(xr.x); v.z += lo_bf16(xr.y); v.w += hi_bf16(xr.y);
                    }
                    *reinterpret_cast<uint2*>(Y + ((long)y * W + x) * C + o) =
                        make_uint2(pack_bf16(fmaxf(v.x, 0.f), fmaxf(v.y, 0.f)), pack_bf16(fmaxf(v.z, 0.f), fmaxf(v.w, 0.f)));
                }
            }
        }
    } else {
        typedef ConvStage<TROW, P2W, TW, P2, G::NMT2> Stage;
        Stage st;
        const bool live = Stage::live(wave);
        const int me = Stage::tg(wave);
        if (live) {
            st.init(wave, j, h);
            st.run(Ts, Ws, h);
        }
        __syncthreads();
        if (live) st.park(reinterpret_cast<float*>(Ws), wave, lane);
        __syncthreads();
        if (live) {
            st.gather(reinterpret_cast<const float*>(Ws), wave, lane);
            // epilogue of the owned groups: lane = pixel, 4 consecutive channels per group: bias, residual,
            // ReLU, 8-byte stores
            const int m = Stage::tile(wave) * 32 + j;
            const int py = m / P2W, px = m % P2W;
            const int y = oh0 + py, x = ow0 + px;
            if (m < P2 && px < TW && y < H && x < W) {
#pragma unroll
                for (int grp = 0; grp < 8; ++grp) {
                    if (Stage::owner_of(grp) != me) continue;
                    const int ot = grp >> 2, g = grp & 3;
                    const int o = ot * 32 + 8 * g + 4 * h;
                    float4 v = make_float4(st.acc[ot][4 * g], st.acc[ot][4 * g + 1], st.acc[ot][4 * g + 2], st.acc[ot][4 * g + 3]);
                    const float4 bv = *reinterpret_cast<const float4*>(Bias + 64 + o);
                    v.x += bv.x; v.y += bv.y; v.z += bv.z; v.w += bv.w;
                    if (residual) {
                        const uint2 xr = *reinterpret_cast<const uint2*>(Xs + (py + 2) * XROW + (px + 2) * LD + o);
                        v.x += lo_bf16(xr.x); v.y += hi_bf16(xr.x); v.z += lo_bf16(xr.y); v.w += hi_bf16(xr.y);
                    }
                    *reinterpret_cast<uint2*>(Y + ((long)y * W + x) * C + o) =
                        make_uint2(pack_bf16(fmaxf(v.x, 0.f), fmaxf(v.y, 0.f)), pack_bf16(fmaxf(v.z, 0.f), fmaxf(v.w, 0.f)));
                }
            }
        }
    }
}

template <int TH, int TW, bool FULL = true>
static hipError_t launch_chain(const void* x, const void* wa, const float* ba, const void* wb,
                               const float* bb, void* y, int N, int H, int W, int residual,
                               hipStream_t s) {
    constexpr size_t smem = ChainGeom<TH, TW>::kSmem;
    static_assert(smem <= 160 * 1024, "LDS");
    auto kern = fused_conv_chain_kernel<TH, TW, FULL>;
    if (hipError_t e = allow_dynamic_lds<fused_conv_chain_kernel<TH, TW, FULL>>((int)((int)smem)); e != hipSuccess) return e;
    const int tiles_h = (H + TH - 1) / TH, tiles_w = (W + TW - 1) / TW;
    prof_start(1, s);
    prof_shape(1, (unsigned)(N * tiles_h * tiles_w), 1024);
    hipLaunchKernelGGL(kern, dim3((unsigned)(N * tiles_h * tiles_w)), dim3(1024), smem, s,
                       (const bf16_t*)x, (const bf16_t*)wa, ba, (const bf16_t*)wb, bb, (bf16_t*)y,
                       H, W, tiles_h, tiles_w, residual);
    prof_stop(1, s);
    return hipGetLastError();
}


// ---------------------------------------------------------------------------------------
// One 3x3 convolution (64 -> 64 channels, zero padding 1) with its epilogue (bias, residual, activation),
// built from the fused kernel's pieces: the same tile geometry, weight staging and matrix loop, reading its
// input tile from global memory instead of computing it.  This is the un-fused operator of Fig. 3 / Fig. 4:
// against the fused chain it differs by the intermediate's trip through memory and by the second launch,
// not by the quality of its inner loop.
// ---------------------------------------------------------------------------------------
template <int TH, int TW>
__global__ __launch_bounds__(1024) void conv3x3_tile_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ Wt, const float* __restrict__ bias,
    const bf16_t* __restrict__ R, bf16_t* __restrict__ Y, int H, int W, int tiles_h, int tiles_w, int act) {
    typedef ChainGeom<TH, TW> G;
    constexpr int C = G::C, LD = G::LD, R1W = G::R1W, P2 = G::P2, TROW = G::TROW, P2W = G::P2W;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* Ts = reinterpret_cast<bf16_t*>(smem);      // [TH + 2][TROW]: the input tile with its one-pixel halo
    bf16_t* Ws = Ts + G::R1H * TROW;                   // [9][64][LD]
    float* Bias = reinterpret_cast<float*>(Ws + 9 * 64 * LD);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 31, h = lane >> 5;
    int b = blockIdx.x;
    const int tw = b % tiles_w; b /= tiles_w;
    const int th = b % tiles_h;
    const int n = b / tiles_h;
    const int oh0 = th * TH, ow0 = tw * TW;
    X += (long)n * H * W * C;
    Y += (long)n * H * W * C;
    if (R) R += (long)n * H * W * C;

    uint2 rw[8], extra[8];
    load_weight_unit(Wt, tid, rw);
    if (tid < 9 * 128 - 1024) load_weight_unit(Wt, 1024 + tid, extra);
    if (tid < 64) Bias[tid] = bias ? bias[tid] : 0.0f;
    for (int it = tid; it < G::R1H * R1W * 8; it += 1024) {
        const int pix = it >> 3, kc = it & 7;
        const int ih = oh0 - 1 + pix / R1W, iw = ow0 - 1 + pix % R1W;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (ih >= 0 && ih < H && iw >= 0 && iw < W) v = ld_u4(X + ((long)ih * W + iw) * C + kc * 8);
        st_u4(Ts + (pix / R1W) * TROW + (pix % R1W) * LD + kc * 8, v);
    }
    store_weight_unit(Ws, tid, rw);
    if (tid < 9 * 128 - 1024) store_weight_unit(Ws, 1024 + tid, extra);
    __syncthreads();

    typedef ConvStageFull<TROW, P2W, TW, P2, G::NMT2> Stage;
    Stage st;
    if (Stage::live(wave)) {
        st.init(wave, j, h);
        st.run(Ts, Ws, h);
        const int m = Stage::tile(wave) * 32 + j;
        const int py = m / P2W, px = m % P2W;
        const int y = oh0 + py, x = ow0 + px;
        if (m < P2 && px < TW && y < H && x < W) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int o = Stage::half(wave) * 32 + 8 * g + 4 * h;
                float4 v = make_float4(st.acc[4 * g], st.acc[4 * g + 1], st.acc[4 * g + 2], st.acc[4 * g + 3]);
                const float4 bv = *reinterpret_cast<const float4*>(Bias + o);
                v.x += bv.x; v.y += bv.y; v.z += bv.z; v.w += bv.w;
                if (R) {
                    const uint2 xr = *reinterpret_cast<const uint2*>(R + ((long)y * W + x) * C + o);
                    v.x += lo_bf16(xr.x); v.y += hi_bf16(xr.x); v.z += lo_bf16(xr.y); v.w += hi_bf16(xr.y);
                }
                *reinterpret_cast<uint2*>(Y + ((long)y * W + x) * C + o) =
                    make_uint2(pack_bf16(apply_act_rt(v.x, act), apply_act_rt(v.y, act)),
                               pack_bf16(apply_act_rt(v.z, act), apply_act_rt(v.w, act)));
            }
        }
    }
}

template <int TH, int TW>
static hipError_t launch_conv3x3_tile(const void* x, const void* w, const float* bias, const void* res, void* y,
                                      int N, int H, int W, int act, hipStream_t s) {
    typedef ChainGeom<TH, TW> G;
    constexpr size_t smem = ((size_t)G::R1H * G::TROW + 9 * 64 * G::LD) * 2 + 64 * 4;
    auto kern = conv3x3_tile_kernel<TH, TW>;
    if (hipError_t e = allow_dynamic_lds<conv3x3_tile_kernel<TH, TW>>((int)smem); e != hipSuccess) return e;
    const int tiles_h = (H + TH - 1) / TH, tiles_w = (W + TW - 1) / TW;
    hipLaunchKernelGGL(kern, dim3((unsigned)(N * tiles_h * tiles_w)), dim3(1024), smem, s, (const bf16_t*)x,
                       (const bf16_t*)w, bias, (const bf16_t*)res, (bf16_t*)y, H, W, tiles_h, tiles_w, act);
    return hipGetLastError();
}

// The un-fused 3x3 convolution: 7 x 14 tiles when they fill the chip, 7 x 7 tiles otherwise (the same
// trade-off the chain's planner makes: more workgroups against more halo pixels loaded).
hipError_t conv3x3_bf16_tiled(const void* x, const void* w, const float* bias, const void* res, void* y,
                              int N, int H, int W, int act, hipStream_t s) {
    const long t714 = (long)N * ((H + 6) / 7) * ((W + 13) / 14);
    if (t714 >= 192) return launch_conv3x3_tile<7, 14>(x, w, bias, res, y, N, H, W, act, s);
    return launch_conv3x3_tile<7, 7>(x, w, bias, res, y, N, H, W, act, s);
}

// Tile configurations (TH x TW output pixels per workgroup): 0: 7x14  1: 7x7  2: 8x8  3: 6x14, each convolution
// cut into (row tile, output-channel half) units; 4: 7x14 and 5: 7x7 with (row tile, kernel row) units, whose
// partial sums meet in LDS (the earlier form, kept for comparison: 12.5 us against 10.9 us on 8 x 56 x 56)
int fused_conv_chain_num_cfgs() { return 6; }

hipError_t fused_conv_chain(const void* x, const void* wa, const float* ba, const void* wb,
                            const float* bb, void* y, int N, int H, int W, int residual, int tile_cfg,
                            hipStream_t s) {
    if (tile_cfg < 0) {        // built-in choice: the candidate the time model predicts fastest
        ChainPlan plan;
        tile_cfg = plan_conv_chain(N, H, W, 64, -1, &plan) ? plan.cfg : 0;
    }
    switch (tile_cfg) {
        case 0: return launch_chain<7, 14>(x, wa, ba, wb, bb, y, N, H, W, residual, s);
        case 1: return launch_chain<7, 7>(x, wa, ba, wb, bb, y, N, H, W, residual, s);
        case 2: return launch_chain<8, 8>(x, wa, ba, wb, bb, y, N, H, W, residual, s);
        case 3: return launch_chain<6, 14>(x, wa, ba, wb, bb, y, N, H, W, residual, s);
        case 4: return launch_chain<7, 14, false>(x, wa, ba, wb, bb, y, N, H, W, residual, s);
        case 5: return launch_chain<7, 7, false>(x, wa, ba, wb, bb, y, N, H, W, residual, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ago
