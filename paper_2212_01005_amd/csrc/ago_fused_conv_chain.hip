// Fused conv3x3 -> conv3x3, 64 -> 64 -> 64 channels, bf16 (AGO Sec. III-B, Fig. 5: a general
// convolution downstream re-uses the upstream result on O2, H2 and W2, so spatial tiling of the
// downstream operator costs recomputation of a one-pixel halo of the upstream operator:
// executed upstream work = ((TH+2)(TW+2)) / (TH TW) of the un-fused count).
//
// One workgroup owns a TH x TW tile of output pixels of one image:
//   load   X tile with a 2-pixel halo, (TH+4) x (TW+4) x 64, zero outside the image -> LDS
//   conv1  T = relu(conv3x3(X) + ba) on the (TH+2) x (TW+2) region -> LDS (bf16), T := 0 outside
//          the image (the intermediate is what the second convolution pads)
//   conv2  Y = relu(conv3x3(T) + bb (+ X)) on TH x TW -> global memory
// Both convolutions are implicit GEMMs [pixels] x [9 taps x 64] x [64] on 32x32x16 bf16 matrix
// instructions.  Weights are streamed one tap (64 x 64) at a time through a double-buffered,
// transposed LDS tile shared by the four waves; waves split the 32-pixel row tiles.
#include "ago_dev.hpp"
#include "ago_launch.hpp"

namespace ago {

template <int TH, int TW>
__global__ __launch_bounds__(256) void fused_conv_chain_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ Wa, const float* __restrict__ ba,
    const bf16_t* __restrict__ Wb, const float* __restrict__ bb, bf16_t* __restrict__ Y,
    int H, int W, int tiles_h, int tiles_w, int residual) {
    constexpr int C = 64, LD = C + 8;
    constexpr int XH = TH + 4, XW = TW + 4, R1H = TH + 2, R1W = TW + 2;
    constexpr int P1 = R1H * R1W, P2 = TH * TW;
    constexpr int NMT1 = (P1 + 31) / 32, NMT2 = (P2 + 31) / 32;
    constexpr int MT1 = (NMT1 + 3) / 4, MT2 = (NMT2 + 3) / 4;   // row tiles per wave
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* Xs = reinterpret_cast<bf16_t*>(smem);      // [XH*XW][LD]
    bf16_t* Ts = Xs + XH * XW * LD;                    // [P1][LD]
    bf16_t* Ws = Ts + P1 * LD;                         // [2][64][LD]  (out channel, in channel)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 31, h = lane >> 5;
    int b = blockIdx.x;
    const int tw = b % tiles_w; b /= tiles_w;
    const int th = b % tiles_h;
    const int n = b / tiles_h;
    const int oh0 = th * TH, ow0 = tw * TW;
    X += (long)n * H * W * C;
    Y += (long)n * H * W * C;

    // weights of one tap: global [c][o] -> registers -> LDS [o][c]
    uint2 rw[8];
    auto load_w = [&](int step) {        // step 0..8: Wa taps, 9..17: Wb taps
        if (tid < 128) {
            const bf16_t* Wt = (step < 9 ? Wa : Wb) + (long)(step % 9) * C * C;
            const int nq = tid & 15, ko = tid >> 4;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk)
                rw[kk] = *reinterpret_cast<const uint2*>(Wt + (ko * 8 + kk) * C + nq * 4);
        }
    };
    auto store_w = [&](int buf) {
        if (tid < 128) {
            const int nq = tid & 15, ko = tid >> 4;
            uint4 t[4];
            transpose_8x4(rw, t);
#pragma unroll
            for (int q = 0; q < 4; ++q) st_u4(Ws + (buf * 64 + nq * 4 + q) * LD + ko * 8, t[q]);
        }
    };

    load_w(0);
    for (int it = tid; it < XH * XW * 8; it += 256) {
        const int pix = it >> 3, kc = it & 7;
        const int ih = oh0 - 2 + pix / XW, iw = ow0 - 2 + pix % XW;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (ih >= 0 && ih < H && iw >= 0 && iw < W) v = ld_u4(X + ((long)ih * W + iw) * C + kc * 8);
        st_u4(Xs + pix * LD + kc * 8, v);
    }
    store_w(0);
    __syncthreads();

    // ---- conv1: rows = output channels (weights are operand A), cols = region pixels ----
    {
        int off[MT1];           // LDS element offset of this lane's pixel (tap 0,0) per row tile
        bool live[MT1];         // wave-uniform: the row tile exists
#pragma unroll
        for (int t = 0; t < MT1; ++t) {
            const int mt = wave + 4 * t;
            live[t] = mt < NMT1;
            int m = mt * 32 + j;
            if (m >= P1) m = 0;
            off[t] = ((m / R1W) * XW + (m % R1W)) * LD + 8 * h;
        }
        f32x16 acc[2][MT1];
        zero_acc(acc);
        for (int tap = 0; tap < 9; ++tap) {
            const int buf = tap & 1;
            load_w(tap + 1);                      // tap 8 prefetches the first tap of conv2
            const int shift = ((tap / 3) * XW + tap % 3) * LD;
            const bf16_t* wsb = Ws + (buf * 64 + j) * LD + 8 * h;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const bf16x8 w0 = ld_bf16x8(wsb + ks * 16), w1 = ld_bf16x8(wsb + 32 * LD + ks * 16);
#pragma unroll
                for (int t = 0; t < MT1; ++t) {
                    if (!live[t]) continue;
                    const bf16x8 xf = ld_bf16x8(Xs + off[t] + shift + ks * 16);
                    acc[0][t] = mfma32(w0, xf, acc[0][t]);
                    acc[1][t] = mfma32(w1, xf, acc[1][t]);
                }
            }
            if (tap == 8) {
                // epilogue: bias + ReLU, zero outside the image, bf16 -> Ts[pixel][channel]
#pragma unroll
                for (int t = 0; t < MT1; ++t) {
                    if (!live[t]) continue;
                    const int m = (wave + 4 * t) * 32 + j;
                    if (m < P1) {
                        const int y = oh0 - 1 + m / R1W, x = ow0 - 1 + m % R1W;
                        const bool inside = y >= 0 && y < H && x >= 0 && x < W;
#pragma unroll
                        for (int ot = 0; ot < 2; ++ot)
#pragma unroll
                            for (int g = 0; g < 4; ++g) {
                                const int o = ot * 32 + 8 * g + 4 * h;
                                uint2 v = make_uint2(0, 0);
                                if (inside) {
                                    float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
                                    if (ba) bv = *reinterpret_cast<const float4*>(ba + o);
                                    v = make_uint2(pack_bf16(fmaxf(acc[ot][t][4 * g] + bv.x, 0.f),
                                                             fmaxf(acc[ot][t][4 * g + 1] + bv.y, 0.f)),
                                                   pack_bf16(fmaxf(acc[ot][t][4 * g + 2] + bv.z, 0.f),
                                                             fmaxf(acc[ot][t][4 * g + 3] + bv.w, 0.f)));
                                }
                                *reinterpret_cast<uint2*>(Ts + m * LD + o) = v;
                            }
                    }
                }
            }
            store_w(buf ^ 1);
            __syncthreads();
        }
    }

    // ---- conv2: rows = output pixels, cols = output channels -------------------------------
    {
        int off[MT2];
        bool live[MT2];
#pragma unroll
        for (int t = 0; t < MT2; ++t) {
            const int mt = wave + 4 * t;
            live[t] = mt < NMT2;
            int m = mt * 32 + j;
            if (m >= P2) m = 0;
            off[t] = ((m / TW) * R1W + (m % TW)) * LD + 8 * h;
        }
        f32x16 acc[MT2][2];
        zero_acc(acc);
        for (int tap = 0; tap < 9; ++tap) {
            const int buf = (tap + 9) & 1;
            if (tap + 1 < 9) load_w(tap + 10);
            const int shift = ((tap / 3) * R1W + tap % 3) * LD;
            const bf16_t* wsb = Ws + (buf * 64 + j) * LD + 8 * h;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const bf16x8 w0 = ld_bf16x8(wsb + ks * 16), w1 = ld_bf16x8(wsb + 32 * LD + ks * 16);
#pragma unroll
                for (int t = 0; t < MT2; ++t) {
                    if (!live[t]) continue;
                    const bf16x8 tf = ld_bf16x8(Ts + off[t] + shift + ks * 16);
                    acc[t][0] = mfma32(tf, w0, acc[t][0]);
                    acc[t][1] = mfma32(tf, w1, acc[t][1]);
                }
            }
            if (tap + 1 < 9) {
                store_w(buf ^ 1);
                __syncthreads();
            }
        }
        // epilogue: lane = output channel, registers = pixels
#pragma unroll
        for (int t = 0; t < MT2; ++t) {
            if (!live[t]) continue;
#pragma unroll
            for (int ot = 0; ot < 2; ++ot) {
                const int o = ot * 32 + j;
                const float bv = bb ? bb[o] : 0.0f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = (wave + 4 * t) * 32 + acc_row(r, h);
                    const int py = m / TW, px = m % TW;
                    const int y = oh0 + py, x = ow0 + px;
                    if (m < P2 && y < H && x < W) {
                        float v = acc[t][ot][r] + bv;
                        if (residual) v += (float)Xs[((py + 2) * XW + px + 2) * LD + o];
                        Y[((long)y * W + x) * C + o] = (bf16_t)fmaxf(v, 0.0f);
                    }
                }
            }
        }
    }
}

template <int TH, int TW>
static hipError_t launch_chain(const void* x, const void* wa, const float* ba, const void* wb,
                               const float* bb, void* y, int N, int H, int W, int residual,
                               hipStream_t s) {
    constexpr size_t smem = ((size_t)(TH + 4) * (TW + 4) + (size_t)(TH + 2) * (TW + 2) + 128) * 72 * 2;
    static_assert(smem <= 160 * 1024, "LDS");
    auto kern = fused_conv_chain_kernel<TH, TW>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles_h = (H + TH - 1) / TH, tiles_w = (W + TW - 1) / TW;
    prof_start(1, s);
    hipLaunchKernelGGL(kern, dim3((unsigned)(N * tiles_h * tiles_w)), dim3(256), smem, s,
                       (const bf16_t*)x, (const bf16_t*)wa, ba, (const bf16_t*)wb, bb, (bf16_t*)y,
                       H, W, tiles_h, tiles_w, residual);
    prof_stop(1, s);
    return hipGetLastError();
}

// Tile configurations (TH x TW output pixels per workgroup): 0: 7x14  1: 14x14  2: 8x8  3: 6x14
int fused_conv_chain_num_cfgs() { return 4; }

hipError_t fused_conv_chain(const void* x, const void* wa, const float* ba, const void* wb,
                            const float* bb, void* y, int N, int H, int W, int residual, int tile_cfg,
                            hipStream_t s) {
    switch (tile_cfg < 0 ? 0 : tile_cfg) {
        case 0: return launch_chain<7, 14>(x, wa, ba, wb, bb, y, N, H, W, residual, s);
        case 1: return launch_chain<14, 14>(x, wa, ba, wb, bb, y, N, H, W, residual, s);
        case 2: return launch_chain<8, 8>(x, wa, ba, wb, bb, y, N, H, W, residual, s);
        case 3: return launch_chain<6, 14>(x, wa, ba, wb, bb, y, N, H, W, residual, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ago
