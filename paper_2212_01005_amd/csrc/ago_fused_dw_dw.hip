// Fused depthwise -> depthwise pair (the dw->dw micro-benchmark of AGO Sec. VI, Fig. 13; both
// operators follow the "downstream depthwise" rule of Sec. III-B / Fig. 7a: a depthwise
// convolution re-uses its input only inside a channel, so a workgroup owns a spatial tile of a
// block of channels and nothing is recomputed except the 1-pixel halo of the intermediate):
//   T = relu6(dw3x3(x, wa, stride) + ba), T := 0 outside its image
//   y = relu6(dw3x3(T, wb, 1) + bb)
// One workgroup = an 8 x 8 tile of output pixels x 32 channels.  The input halo tile and the
// 10 x 10 intermediate region live in LDS as fp32; all arithmetic is on the vector ALUs (a
// depthwise convolution has no reduction over channels, so the matrix cores have nothing to do).
#include "ago_dev.hpp"
#include "ago_launch.hpp"

namespace ago {
namespace {

constexpr int kDwTH = 8, kDwTW = 8, kDwCB = 32, kDwThreads = 256;

template <bool BF16>
__device__ __forceinline__ float4 load_quad(const void* base, long idx) {
    if constexpr (BF16) {
        const uint2 u = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(base) + idx);
        return make_float4(lo_bf16(u.x), hi_bf16(u.x), lo_bf16(u.y), hi_bf16(u.y));
    } else {
        return *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + idx);
    }
}

template <bool BF16, int STRIDE>
__global__ __launch_bounds__(kDwThreads) void fused_dw_dw_kernel(
    const void* __restrict__ x, const void* __restrict__ wa, const float* __restrict__ ba,
    const void* __restrict__ wb, const float* __restrict__ bb, void* __restrict__ y,
    int H, int W, int C, int OH, int OW, int tiles_h, int tiles_w, int cblocks) {
    constexpr int RH = kDwTH + 2, RW = kDwTW + 2;                          // intermediate region
    constexpr int IH = (RH - 1) * STRIDE + 3, IW = (RW - 1) * STRIDE + 3;  // input halo tile
    constexpr int Q = kDwCB / 4;
    extern __shared__ __align__(16) unsigned char smem[];
    float4* Xs = reinterpret_cast<float4*>(smem);          // [IH*IW][Q]
    float4* Ts = Xs + IH * IW * Q;                         // [RH*RW][Q]
    float4* Wa = Ts + RH * RW * Q;                         // [9][Q]
    float4* Wb = Wa + 9 * Q;                               // [9][Q]
    float4* Ba = Wb + 9 * Q;                               // [Q]
    float4* Bb = Ba + Q;                                   // [Q]

    const int tid = threadIdx.x;
    int b = blockIdx.x;
    const int cb = b % cblocks; b /= cblocks;
    const int tw = b % tiles_w; b /= tiles_w;
    const int th = b % tiles_h;
    const int n = b / tiles_h;
    const int c0 = cb * kDwCB;
    const int nq = min(Q, (C - c0) / 4);                   // channel quads of this block that exist
    const int oh0 = th * kDwTH, ow0 = tw * kDwTW;
    const int ih0 = (oh0 - 1) * STRIDE - 1, iw0 = (ow0 - 1) * STRIDE - 1;
    const long xbase = (long)n * H * W * C;

    const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int it = tid; it < 9 * Q; it += kDwThreads) {
        const int q = it % Q, tap = it / Q;
        Wa[it] = q < nq ? load_quad<BF16>(wa, (long)tap * C + c0 + 4 * q) : zero;
        Wb[it] = q < nq ? load_quad<BF16>(wb, (long)tap * C + c0 + 4 * q) : zero;
    }
    if (tid < Q) {
        Ba[tid] = (ba && tid < nq) ? *reinterpret_cast<const float4*>(ba + c0 + 4 * tid) : zero;
        Bb[tid] = (bb && tid < nq) ? *reinterpret_cast<const float4*>(bb + c0 + 4 * tid) : zero;
    }
    for (int it = tid; it < IH * IW * Q; it += kDwThreads) {
        const int q = it % Q, pix = it / Q;
        const int ih = ih0 + pix / IW, iw = iw0 + pix % IW;
        float4 v = zero;
        if (q < nq && ih >= 0 && ih < H && iw >= 0 && iw < W)
            v = load_quad<BF16>(x, xbase + ((long)ih * W + iw) * C + c0 + 4 * q);
        Xs[it] = v;
    }
    __syncthreads();

    // intermediate region: pixel (ty, tx) is T[oh0 - 1 + ty][ow0 - 1 + tx]
    for (int it = tid; it < RH * RW * Q; it += kDwThreads) {
        const int q = it % Q, pix = it / Q;
        const int ty = pix / RW, tx = pix % RW;
        const int gy = oh0 - 1 + ty, gx = ow0 - 1 + tx;
        float4 a = zero;
        if (gy >= 0 && gy < OH && gx >= 0 && gx < OW) {
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int s = 0; s < 3; ++s) {
                    const float4 e = Xs[((ty * STRIDE + r) * IW + tx * STRIDE + s) * Q + q];
                    const float4 w = Wa[(r * 3 + s) * Q + q];
                    a.x = fmaf(e.x, w.x, a.x); a.y = fmaf(e.y, w.y, a.y);
                    a.z = fmaf(e.z, w.z, a.z); a.w = fmaf(e.w, w.w, a.w);
                }
            const float4 bv = Ba[q];
            a.x = apply_act<kRelu6>(a.x + bv.x); a.y = apply_act<kRelu6>(a.y + bv.y);
            a.z = apply_act<kRelu6>(a.z + bv.z); a.w = apply_act<kRelu6>(a.w + bv.w);
        }
        Ts[it] = a;
    }
    __syncthreads();

    for (int it = tid; it < kDwTH * kDwTW * Q; it += kDwThreads) {
        const int q = it % Q, pix = it / Q;
        const int oy = pix / kDwTW, ox = pix % kDwTW;
        const int oh = oh0 + oy, ow = ow0 + ox;
        if (q >= nq || oh >= OH || ow >= OW) continue;
        float4 a = zero;
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                const float4 e = Ts[((oy + r) * RW + ox + s) * Q + q];
                const float4 w = Wb[(r * 3 + s) * Q + q];
                a.x = fmaf(e.x, w.x, a.x); a.y = fmaf(e.y, w.y, a.y);
                a.z = fmaf(e.z, w.z, a.z); a.w = fmaf(e.w, w.w, a.w);
            }
        const float4 bv = Bb[q];
        a.x = apply_act<kRelu6>(a.x + bv.x); a.y = apply_act<kRelu6>(a.y + bv.y);
        a.z = apply_act<kRelu6>(a.z + bv.z); a.w = apply_act<kRelu6>(a.w + bv.w);
        const long o = (((long)n * OH + oh) * OW + ow) * C + c0 + 4 * q;
        if constexpr (BF16) {
            *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(y) + o) = make_uint2(pack_bf16(a.x, a.y), pack_bf16(a.z, a.w));
        } else {
            *reinterpret_cast<float4*>(reinterpret_cast<float*>(y) + o) = a;
        }
    }
}

template <bool BF16, int STRIDE>
hipError_t launch_dw_dw(const void* x, const void* wa, const float* ba, const void* wb, const float* bb,
                        void* y, int N, int H, int W, int C, hipStream_t s) {
    constexpr int RH = kDwTH + 2, RW = kDwTW + 2, IH = (RH - 1) * STRIDE + 3, IW = (RW - 1) * STRIDE + 3;
    constexpr int Q = kDwCB / 4;
    constexpr size_t smem = (size_t)(IH * IW + RH * RW + 18 + 2) * Q * 16;
    static_assert(smem <= 160 * 1024, "LDS");
    auto kern = fused_dw_dw_kernel<BF16, STRIDE>;
    if (hipError_t e = allow_dynamic_lds<fused_dw_dw_kernel<BF16, STRIDE>>((int)((int)smem)); e != hipSuccess) return e;
    const int OH = (H - 1) / STRIDE + 1, OW = (W - 1) / STRIDE + 1;
    const int tiles_h = (OH + kDwTH - 1) / kDwTH, tiles_w = (OW + kDwTW - 1) / kDwTW;
    const int cblocks = (C + kDwCB - 1) / kDwCB;
    const long grid = (long)N * tiles_h * tiles_w * cblocks;
    if (grid >= (1L << 31)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kDwThreads), smem, s, x, wa, ba, wb, bb, y, H, W, C, OH, OW,
                       tiles_h, tiles_w, cblocks);
    return hipGetLastError();
}

}  // namespace

hipError_t fused_dw_dw(const void* x, const void* wa, const float* ba, const void* wb, const float* bb,
                       void* y, int N, int H, int W, int C, int stride, bool bf16, hipStream_t s) {
    if (bf16) return stride == 1 ? launch_dw_dw<true, 1>(x, wa, ba, wb, bb, y, N, H, W, C, s)
                                 : launch_dw_dw<true, 2>(x, wa, ba, wb, bb, y, N, H, W, C, s);
    return stride == 1 ? launch_dw_dw<false, 1>(x, wa, ba, wb, bb, y, N, H, W, C, s)
                       : launch_dw_dw<false, 2>(x, wa, ba, wb, bb, y, N, H, W, C, s);
}

}  // namespace ago
