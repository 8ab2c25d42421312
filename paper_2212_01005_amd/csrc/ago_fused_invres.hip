// Fused pointwise -> depthwise -> pointwise block (AGO Sec. III-B: pw->dw follows the
// "downstream depthwise" rule of Fig. 7a, dw->pw the "downstream pointwise" rule of Fig. 7b).
//
// One workgroup owns a TOH x TOW tile of output pixels of one image and *all* expanded
// channels, so the depthwise stage needs no data from other workgroups and the projection
// reduces over channels that are all on-chip.  The expanded tensor E for the tile plus its
// halo of (KS - 1) / 2 pixels (recomputed by neighbouring tiles) lives in LDS as fp32; the depthwise output D
// lives in LDS in the matrix-instruction input type.  Stages, separated by workgroup barriers:
//   0  global -> LDS: X halo tile, W1, Wd, W2 (weights transposed for the bf16 path)
//   1  E = relu6(X W1 + b1) on the matrix cores; E := 0 for pixels outside the image
//   2  D = relu6(dw KSxKS(E) + bd) on the vector ALUs (KS = 3, or 5 as in MNasNet-style blocks)
//   3  Y = D W2 + b2 (+ X) on the matrix cores, stored straight to global memory
// Matrix instructions: 16x16x32 bf16 / 16x16x4 fp32 (small tiles: few pixels per workgroup).
//
// When the weights and E of all expanded channels do not fit LDS (the 576- and 960-channel blocks
// of the networks), stages 0-3 run once per chunk of CC expanded channels: the projection reduces over
// the expanded channels, so each chunk adds its slice of that reduction to accumulators that stay
// in registers (the "downstream pointwise" rule applied inside the block: D is consumed in slices
// of the reduction dimension).  One chunk = the whole of Cexp is the common case.
//
// Channel split (SPLIT): a wide block on few pixels (the 7 x 7 x 960 blocks at batch 1 are one tile)
// leaves most of the chip idle if one workgroup walks all the chunks.  With a workspace the chunks go
// to different workgroups instead (grid.y = chunk): each runs stages 0-3 for its chunk and writes its
// slice of the projection's reduction as an fp32 partial; invres_reduce_kernel adds the partials, b2
// and the residual.  Same rule as above, with the slices of the reduction spread over the chip.
//
// The same kernel runs the two-operator pairs of the block (the paper's Fig. 13 micro-benchmarks):
//   mode 1  pw -> dw: stages 0-2, D is stored to global memory instead of LDS
//   mode 2  dw -> pw: the input *is* E (stage 0 loads its halo tile into the E region, zero outside
//           the image), stages 2-3 follow
#include "ago_dev.hpp"
#include "ago_launch.hpp"
#include <utility>

namespace ago {

struct InvresParams {
    const void* x; const void* w1; const float* b1; const void* wd; const float* bd;
    const void* w2; const float* b2; void* y;
    int N, H, W, Cin, Cexp, Cout, OH, OW, residual;
    int TOH, TOW, tiles_h, tiles_w;
    int EH, EW, PE, PEpad, POpad;   // E-region geometry of one tile
    int KP1;                        // Cin padded to the k granularity of the matrix instruction
    int CC, nchunks;                // expanded channels per chunk (multiple of 16), number of chunks
    int KPC;                        // CC padded to the k granularity
    int CoutP;                      // Cout padded to 16
    int ldx, ldw1, lde, ldd, ldw2;  // LDS leading dimensions (elements)
    int off_w1, off_e, off_d, off_w2, off_wd, off_b;  // LDS byte offsets (Xs at 0)
    int ksplit;                     // stage 3: waves per (pixel tile, channel tile) job, splitting k
    int mode;                       // 0: pw -> dw -> pw   1: pw -> dw   2: dw -> pw
    int nsplit;                     // channel split: workgroups per tile (one chunk each), 1 = none
    float* part;                    // channel split: [nsplit][N][OH][OW][Cout] fp32 partial projections
};

template <bool BF16> struct InT { typedef float type; };
template <> struct InT<true> { typedef bf16_t type; };

constexpr int kInvresThreads = 1024;   // 16 waves: LDS / global latency is hidden by wave-level parallelism
constexpr int kInvresWaves = kInvresThreads / 64;
constexpr int kInvresJobsPerWave = 4;  // stage-3 accumulators a wave can hold across the chunks

static constexpr int round_up(int v, int m) { return (v + m - 1) / m * m; }

// Lay out LDS for a tile and a chunk width cc of expanded channels; returns the byte count.
static constexpr size_t plan_layout(InvresParams& p, bool bf16, int stride, int toh, int tow, int ksize, int cc) {
    p.TOH = toh; p.TOW = tow;
    p.tiles_h = (p.OH + toh - 1) / toh; p.tiles_w = (p.OW + tow - 1) / tow;
    p.EH = (toh - 1) * stride + ksize; p.EW = (tow - 1) * stride + ksize;
    p.PE = p.EH * p.EW; p.PEpad = round_up(p.PE, 16); p.POpad = round_up(toh * tow, 16);
    const int kg = bf16 ? 32 : 4, es = bf16 ? 2 : 4;
    p.CC = cc; p.nchunks = (p.Cexp + cc - 1) / cc;
    p.KP1 = round_up(p.Cin, kg); p.KPC = round_up(cc, kg); p.CoutP = round_up(p.Cout, 16);
    auto pad16 = [](int c) { int q = c; while (q % 32 != 16) q += 4; return q; };  // fp32 [k][n] rows
    p.ldx = bf16 ? p.KP1 + 8 : p.KP1 + 4;
    p.ldw1 = bf16 ? p.KP1 + 8 : pad16(cc);
    p.lde = cc + 4;
    p.ldd = bf16 ? p.KPC + 8 : p.KPC + 4;
    p.ldw2 = bf16 ? p.KPC + 8 : pad16(p.CoutP);
    size_t off = (size_t)p.PEpad * p.ldx * es;
    auto al = [](size_t v) { return (v + 15) / 16 * 16; };
    p.off_w1 = (int)(off = al(off));
    off += (size_t)(bf16 ? cc : p.KP1) * p.ldw1 * es;
    p.off_e = (int)(off = al(off));
    off += (size_t)p.PE * p.lde * 4;
    p.off_d = (int)(off = al(off));
    off += (size_t)p.POpad * p.ldd * es;
    p.off_w2 = (int)(off = al(off));
    off += (size_t)(bf16 ? p.CoutP : p.KPC) * p.ldw2 * es;
    p.off_wd = (int)(off = al(off));
    off += (size_t)ksize * ksize * cc * 4;
    p.off_b = (int)(off = al(off));
    off += (size_t)(2 * p.Cexp + p.CoutP) * 4;
    // stage-3 k split: as many waves per job as there are, limited by the k steps of a chunk and by
    // the scratch (1 KB per wave) that fits in the E region
    const int njobs = (p.POpad / 16) * (p.CoutP / 16);
    const int ksteps = p.KPC / kg;
    int ks = njobs < kInvresWaves ? kInvresWaves / njobs : 1;
    if (ks > ksteps) ks = ksteps;
    const size_t e_bytes = (size_t)p.PE * p.lde * 4;
    while (ks > 1 && (size_t)njobs * ks * 1024 > e_bytes) --ks;
    p.ksplit = ks < 1 ? 1 : ks;
    return al(off);
}

// Shape-specialised instantiations: the paper's tuner emits code for one subgraph shape at a time, so tile sizes,
// strides and trip counts are constants of the generated loop nest.  SPEC > 0 selects a geometry known at
// compile time (all integer fields of the parameter block, laid out by the same plan_layout as at run time):
// index arithmetic by constants, fully unrolled job loops, dead modes removed.  The launcher picks such an
// instantiation only when the run-time plan is field for field the same.
// The table: the two benchmark blocks, the eleven block shapes of a MobileNetV2-style network at batch 1 and the
// two-operator pairs of the benchmark blocks, each with the tile (and, for the wide blocks, the channel split)
// the planner picks for it.
struct InvresSpecShape { int N, H, W, Cin, Cexp, Cout, stride, bf16, residual, toh, tow, cc, split, mode; };
constexpr InvresSpecShape kInvresSpecs[] = {
    {},
    {1, 14, 14, 32, 192, 32, 1, 0, 1, 2, 2, 192, 0},       // benchmark block, fp32
    {1, 56, 56, 24, 144, 32, 2, 1, 0, 2, 2, 144, 0},       // benchmark block, bf16 (= the network's 56 x 56 stride-2 block)
    {1, 112, 112, 16, 96, 24, 2, 1, 0, 2, 7, 96, 0},
    {1, 56, 56, 24, 144, 24, 1, 1, 1, 4, 4, 144, 0},
    {1, 28, 28, 32, 192, 32, 1, 1, 1, 2, 2, 192, 0},
    {1, 28, 28, 32, 192, 64, 2, 1, 0, 1, 2, 192, 0},
    {1, 14, 14, 64, 384, 64, 1, 1, 1, 1, 1, 384, 0},
    {1, 14, 14, 64, 384, 96, 1, 1, 0, 2, 3, 64, 1},
    {1, 14, 14, 96, 576, 96, 1, 1, 1, 2, 3, 96, 1},
    {1, 14, 14, 96, 576, 160, 2, 1, 0, 1, 2, 64, 1},
    {1, 7, 7, 160, 960, 160, 1, 1, 1, 2, 2, 64, 1},
    {1, 7, 7, 160, 960, 320, 1, 1, 0, 2, 2, 64, 1},
    // the pw -> dw and dw -> pw pairs cut from the two benchmark blocks (mode 1: Cout unused, 16; mode 2: Cin unused, 8)
    {1, 14, 14, 32, 192, 16, 1, 0, 0, 1, 1, 192, 0, 1},
    {1, 56, 56, 24, 144, 16, 2, 1, 0, 2, 2, 144, 0, 1},
    {1, 14, 14, 8, 192, 32, 1, 0, 0, 1, 1, 192, 0, 2},
    {1, 56, 56, 8, 144, 32, 2, 1, 0, 2, 2, 144, 0, 2},
};
constexpr int kNumInvresSpecs = (int)(sizeof(kInvresSpecs) / sizeof(kInvresSpecs[0]));
constexpr InvresParams invres_spec_geometry(int spec) {
    const InvresSpecShape q = kInvresSpecs[spec];
    InvresParams p = {};
    p.N = q.N; p.H = q.H; p.W = q.W; p.Cin = q.Cin; p.Cexp = q.Cexp; p.Cout = q.Cout;
    p.OH = (q.H - 1) / q.stride + 1; p.OW = (q.W - 1) / q.stride + 1;
    p.residual = q.residual; p.mode = q.mode;
    plan_layout(p, q.bf16 != 0, q.stride, q.toh, q.tow, 3, q.cc);
    p.nsplit = q.split ? p.nchunks : 1;
    return p;
}
// true when the run-time parameter block has exactly the geometry of specialisation `spec`
inline bool invres_matches_spec(const InvresParams& a, int spec) {
    const InvresParams b = invres_spec_geometry(spec);
    return a.N == b.N && a.H == b.H && a.W == b.W && a.Cin == b.Cin && a.Cexp == b.Cexp && a.Cout == b.Cout && a.OH == b.OH &&
           a.OW == b.OW && a.residual == b.residual && a.TOH == b.TOH && a.TOW == b.TOW && a.tiles_h == b.tiles_h &&
           a.tiles_w == b.tiles_w && a.EH == b.EH && a.EW == b.EW && a.PE == b.PE && a.PEpad == b.PEpad && a.POpad == b.POpad &&
           a.KP1 == b.KP1 && a.CC == b.CC && a.nchunks == b.nchunks && a.KPC == b.KPC && a.CoutP == b.CoutP && a.ldx == b.ldx &&
           a.ldw1 == b.ldw1 && a.lde == b.lde && a.ldd == b.ldd && a.ldw2 == b.ldw2 && a.off_w1 == b.off_w1 && a.off_e == b.off_e &&
           a.off_d == b.off_d && a.off_w2 == b.off_w2 && a.off_wd == b.off_wd && a.off_b == b.off_b && a.ksplit == b.ksplit &&
           a.mode == b.mode && a.nsplit == b.nsplit;
}

// KS: odd depthwise kernel size (3 or 5), zero padding (KS - 1) / 2.  CHUNKED: several chunks of expanded
// channels with the projection's accumulators carried in registers; the single-chunk instantiation
// keeps none (64 registers or fewer: two workgroups per compute unit).  SPLIT (single-chunk only): the
// workgroup's chunk is blockIdx.y and the projection's partial goes to the workspace.
template <bool BF16, int STRIDE, int KS, bool CHUNKED, bool SPLIT = false, int SPEC = 0>
__global__ __launch_bounds__(kInvresThreads) void fused_invres_kernel(const InvresParams p_in) {
    typedef typename InT<BF16>::type T;
    InvresParams p = p_in;
    if constexpr (SPEC != 0) {
        constexpr InvresParams G = invres_spec_geometry(SPEC);
        p = G;
        p.x = p_in.x; p.w1 = p_in.w1; p.b1 = p_in.b1; p.wd = p_in.wd; p.bd = p_in.bd; p.w2 = p_in.w2; p.b2 = p_in.b2;
        p.y = p_in.y; p.part = p_in.part;
    }
    extern __shared__ __align__(16) unsigned char smem[];
    T* Xs = reinterpret_cast<T*>(smem);
    T* W1s = reinterpret_cast<T*>(smem + p.off_w1);
    float* Es = reinterpret_cast<float*>(smem + p.off_e);
    T* Ds = reinterpret_cast<T*>(smem + p.off_d);
    T* W2s = reinterpret_cast<T*>(smem + p.off_w2);
    float* Wds = reinterpret_cast<float*>(smem + p.off_wd);     // [KS * KS][CC]
    float* B1s = reinterpret_cast<float*>(smem + p.off_b);      // b1[Cexp], bd[Cexp], b2[CoutP]; 0 when absent
    float* Bds = B1s + p.Cexp;
    float* B2s = Bds + p.Cexp;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, g = lane >> 4;
    int b = blockIdx.x;
    const int tw = b % p.tiles_w; b /= p.tiles_w;
    const int th = b % p.tiles_h;
    const int n = b / p.tiles_h;
    const int oh0 = th * p.TOH, ow0 = tw * p.TOW;
    constexpr int PAD = (KS - 1) / 2;
    const int ih0 = oh0 * STRIDE - PAD, iw0 = ow0 * STRIDE - PAD;
    const T* X = reinterpret_cast<const T*>(p.x) + (long)n * p.H * p.W * p.Cin;
    constexpr int VE = BF16 ? 8 : 4;   // elements per 16-byte chunk
    constexpr int KG = BF16 ? 32 : 4;  // k per matrix instruction

    // ---- stage 0 (once): the X halo tile and the biases ---------------------------------
    if (p.mode != 2) {
        const int kch = p.KP1 / VE;
        for (int it = tid; it < p.PEpad * kch; it += kInvresThreads) {
            const int pix = it / kch, kc = it % kch;
            const int ey = pix / p.EW, ex = pix % p.EW;
            const int ih = ih0 + ey, iw = iw0 + ex;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (pix < p.PE && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W && kc * VE < p.Cin)
                v = ld_u4(X + ((long)ih * p.W + iw) * p.Cin + kc * VE);
            st_u4(Xs + pix * p.ldx + kc * VE, v);
        }
    }
    for (int it = tid; it < 2 * p.Cexp + p.CoutP; it += kInvresThreads) {
        float v = 0.0f;
        if (it < p.Cexp) { if (p.b1) v = p.b1[it]; }
        else if (it < 2 * p.Cexp) { if (p.bd) v = p.bd[it - p.Cexp]; }
        else if (it - 2 * p.Cexp < p.Cout) { if (p.b2) v = p.b2[it - 2 * p.Cexp]; }
        B1s[it] = v;
    }

    // stage-3 accumulators: job = wave + 16 jj without a k split, job = wave / ksplit with one
    const int ptiles3 = p.POpad / 16, njobs = ptiles3 * (p.CoutP / 16);
    f32x4 accj[CHUNKED ? kInvresJobsPerWave : 1];
#pragma unroll
    for (int jj = 0; jj < (CHUNKED ? kInvresJobsPerWave : 1); ++jj) accj[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
    static_assert(!(SPLIT && CHUNKED), "a split workgroup runs one chunk");
    T* Y = reinterpret_cast<T*>(p.y) + (long)n * p.OH * p.OW * p.Cout;
    float* P = SPLIT ? p.part + ((long)blockIdx.y * p.N + n) * p.OH * p.OW * p.Cout : nullptr;
    auto emit = [&](int pt, int ot, const f32x4& acc) {
        const int co = ot * 16 + i;        // this lane's output channel; registers = pixels 4g..4g+3
        if (co >= p.Cout) return;
        const float bv = B2s[co];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int po = pt * 16 + 4 * g + r;
            const int oy = po / p.TOW, ox = po % p.TOW;
            const int oh = oh0 + oy, ow = ow0 + ox;
            if (po < p.TOH * p.TOW && oh < p.OH && ow < p.OW) {
                if constexpr (SPLIT) {
                    P[((long)oh * p.OW + ow) * p.Cout + co] = acc[r];
                } else {
                    float v = acc[r] + bv;
                    if (p.residual) v += (float)Xs[((oy + PAD) * p.EW + ox + PAD) * p.ldx + co];
                    Y[((long)oh * p.OW + ow) * p.Cout + co] = (T)v;
                }
            }
        }
    };

    const int nchunks = CHUNKED ? p.nchunks : 1;
    for (int chunk = 0; chunk < nchunks; ++chunk) {
        const int c0 = (SPLIT ? (int)blockIdx.y : chunk) * p.CC;   // first expanded channel of the chunk
        const int cw = min(p.CC, p.Cexp - c0);             // its width (a multiple of 16)
        const int kpc = (cw + KG - 1) / KG * KG;           // padded to the k granularity (zeros beyond cw)

        // ---- stage 0 (per chunk): weights of the chunk, and E itself for dw -> pw ---------
        if (p.mode == 2) {
            // the input has Cexp channels and is the depthwise operand itself: fp32 into the E region
            const T* Xe = reinterpret_cast<const T*>(p.x) + (long)n * p.H * p.W * p.Cexp + c0;
            const int q4 = cw / 4;
            for (int it = tid; it < p.PE * q4; it += kInvresThreads) {
                const int pix = it / q4, q = it % q4;
                const int ih = ih0 + pix / p.EW, iw = iw0 + pix % p.EW;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (ih >= 0 && ih < p.H && iw >= 0 && iw < p.W) {
                    const T* src = Xe + ((long)ih * p.W + iw) * p.Cexp + 4 * q;
                    if constexpr (BF16) {
                        const uint2 u = *reinterpret_cast<const uint2*>(src);
                        v = make_float4(lo_bf16(u.x), hi_bf16(u.x), lo_bf16(u.y), hi_bf16(u.y));
                    } else {
                        v = *reinterpret_cast<const float4*>(src);
                    }
                }
                *reinterpret_cast<float4*>(Es + pix * p.lde + 4 * q) = v;
            }
        }
        if constexpr (BF16) {
            // W1 [Cin][Cexp] -> W1s[e][k], W2 [Cexp][Cout] -> W2s[co][k]; k beyond the real extent = 0
            const bf16_t* W1 = reinterpret_cast<const bf16_t*>(p.w1) + c0;
            const int nq1 = p.mode == 2 ? 0 : cw / 4;
            // unit = (8 input channels ko, 4 output channels nq).  Sixteen consecutive threads take (nq & 3, ko & 3),
            // nq fastest: a quad of lanes loads 32 contiguous bytes of a weight row, and because the rows of W1s /
            // W2s are an odd number c of 16-byte chunks long, the 16 lanes that a 16-byte LDS store serves
            // together hit 16 different chunks (4 c (nq & 3) + (ko & 3) mod 16)
            for (int it = tid; it < (p.KP1 / 8) * nq1; it += kInvresThreads) {
                const int hi = it >> 4, nq = (hi % (nq1 / 4)) * 4 + (it & 3), ko = (hi / (nq1 / 4)) * 4 + ((it >> 2) & 3);
                uint2 r[8];
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    const int k = ko * 8 + kk;
                    r[kk] = k < p.Cin ? *reinterpret_cast<const uint2*>(W1 + (long)k * p.Cexp + nq * 4) : make_uint2(0, 0);
                }
                uint4 t[4];
                transpose_8x4(r, t);
#pragma unroll
                for (int q = 0; q < 4; ++q) st_u4(W1s + (nq * 4 + q) * p.ldw1 + ko * 8, t[q]);
            }
            const bf16_t* W2 = reinterpret_cast<const bf16_t*>(p.w2) + (long)c0 * p.Cout;
            const int nq2 = p.mode == 1 ? 0 : p.CoutP / 4;
            for (int it = tid; it < (kpc / 8) * nq2; it += kInvresThreads) {
                const int hi = it >> 4, nq = (hi % (nq2 / 4)) * 4 + (it & 3), ko = (hi / (nq2 / 4)) * 4 + ((it >> 2) & 3);
                uint2 r[8];
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    const int k = ko * 8 + kk;
                    r[kk] = (k < cw && nq * 4 < p.Cout)
                                ? *reinterpret_cast<const uint2*>(W2 + (long)k * p.Cout + nq * 4) : make_uint2(0, 0);
                }
                uint4 t[4];
                transpose_8x4(r, t);
#pragma unroll
                for (int q = 0; q < 4; ++q) st_u4(W2s + (nq * 4 + q) * p.ldw2 + ko * 8, t[q]);
            }
            // depthwise weights as fp32 [KS * KS][CC]
            const uint16_t* WD = reinterpret_cast<const uint16_t*>(p.wd) + c0;
            for (int it = tid; it < KS * KS * cw; it += kInvresThreads) {
                const int tap = it / cw, ch = it % cw;
                Wds[tap * p.CC + ch] = bf16_to_f32(WD[tap * p.Cexp + ch]);
            }
        } else {
            // fp32: weights keep their [k][n] layout (the fp32 matrix instruction reads one k per lane)
            const float* W1 = reinterpret_cast<const float*>(p.w1) + c0;
            const int c4 = p.mode == 2 ? 0 : cw / 4;
            for (int it = tid; it < p.KP1 * c4; it += kInvresThreads) {
                const int k = it / c4, q = it % c4;
                const uint4 v = k < p.Cin ? ld_u4(W1 + (long)k * p.Cexp + q * 4) : make_uint4(0, 0, 0, 0);
                st_u4(W1s + k * p.ldw1 + q * 4, v);
            }
            const float* W2 = reinterpret_cast<const float*>(p.w2) + (long)c0 * p.Cout;
            const int o4 = p.mode == 1 ? 0 : p.CoutP / 4;
            for (int it = tid; it < kpc * o4; it += kInvresThreads) {
                const int k = it / o4, q = it % o4;
                const uint4 v = (k < cw && q * 4 < p.Cout) ? ld_u4(W2 + (long)k * p.Cout + q * 4)
                                                          : make_uint4(0, 0, 0, 0);
                st_u4(W2s + k * p.ldw2 + q * 4, v);
            }
            const float* WD = reinterpret_cast<const float*>(p.wd) + c0;
            for (int it = tid; it < KS * KS * cw; it += kInvresThreads) {
                const int tap = it / cw, ch = it % cw;
                Wds[tap * p.CC + ch] = WD[tap * p.Cexp + ch];
            }
        }
        __syncthreads();

        // ---- stage 1: expand.  acc rows = channels, cols = pixels (weights are operand A) ---
        if (p.mode != 2) {
            const int ptiles = p.PEpad / 16, ctiles = cw / 16;
            for (int job = wave; job < ptiles * ctiles; job += kInvresWaves) {
                const int pt = job % ptiles, ct = job / ptiles;
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                if constexpr (BF16) {
                    const bf16_t* ap = W1s + (ct * 16 + i) * p.ldw1 + 8 * g;
                    const bf16_t* bp = Xs + (pt * 16 + i) * p.ldx + 8 * g;
                    for (int k0 = 0; k0 < p.KP1; k0 += 32)
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ld_bf16x8(ap + k0), ld_bf16x8(bp + k0), acc, 0, 0, 0);
                } else {
                    const float* ap = W1s + g * p.ldw1 + ct * 16 + i;
                    const float* bp = Xs + (pt * 16 + i) * p.ldx + g;
#pragma unroll 8
                    for (int k0 = 0; k0 < p.KP1; k0 += 4)
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ap[k0 * p.ldw1], bp[k0], acc, 0, 0, 0);
                }
                const int pix = pt * 16 + i;       // this lane's pixel; registers = channels 4g..4g+3
                if (pix < p.PE) {
                    const int ey = pix / p.EW, ex = pix % p.EW;
                    const int ih = ih0 + ey, iw = iw0 + ex;
                    const bool inside = ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
                    const int e0 = ct * 16 + 4 * g;
                    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (inside) {
                        const float4 bv = *reinterpret_cast<const float4*>(B1s + c0 + e0);
                        v.x = apply_act<kRelu6>(acc[0] + bv.x);
                        v.y = apply_act<kRelu6>(acc[1] + bv.y);
                        v.z = apply_act<kRelu6>(acc[2] + bv.z);
                        v.w = apply_act<kRelu6>(acc[3] + bv.w);
                    }
                    *reinterpret_cast<float4*>(Es + pix * p.lde + e0) = v;
                }
            }
        }
        __syncthreads();

        // ---- stage 2: depthwise KS x KS on the vector ALUs -----------------------------------
        {
            const int Q = kpc / 4;             // channel quads including the zero k-padding of D
            const int Qr = cw / 4;
            for (int it = tid; it < p.TOH * p.TOW * Q; it += kInvresThreads) {
                const int q = it % Q, po = it / Q;
                float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
                if (q < Qr) {
                    const int oy = po / p.TOW, ox = po % p.TOW;
                    const float* ep = Es + ((oy * STRIDE) * p.EW + ox * STRIDE) * p.lde + 4 * q;
#pragma unroll
                    for (int r = 0; r < KS; ++r)
#pragma unroll
                        for (int s = 0; s < KS; ++s) {
                            const float4 e = *reinterpret_cast<const float4*>(ep + (r * p.EW + s) * p.lde);
                            const float4 w = *reinterpret_cast<const float4*>(Wds + (r * KS + s) * p.CC + 4 * q);
                            a.x = fmaf(e.x, w.x, a.x); a.y = fmaf(e.y, w.y, a.y);
                            a.z = fmaf(e.z, w.z, a.z); a.w = fmaf(e.w, w.w, a.w);
                        }
                    const float4 bv = *reinterpret_cast<const float4*>(Bds + c0 + 4 * q);
                    a.x = apply_act<kRelu6>(a.x + bv.x); a.y = apply_act<kRelu6>(a.y + bv.y);
                    a.z = apply_act<kRelu6>(a.z + bv.z); a.w = apply_act<kRelu6>(a.w + bv.w);
                }
                T* dst = Ds + po * p.ldd + 4 * q;
                if (p.mode == 1) {                 // pw -> dw: D is the result
                    const int oh = oh0 + po / p.TOW, ow = ow0 + po % p.TOW;
                    if (q >= Qr || oh >= p.OH || ow >= p.OW) continue;
                    dst = reinterpret_cast<T*>(p.y) + (((long)n * p.OH + oh) * p.OW + ow) * p.Cexp + c0 + 4 * q;
                }
                if constexpr (BF16) {
                    *reinterpret_cast<uint2*>(dst) = make_uint2(pack_bf16(a.x, a.y), pack_bf16(a.z, a.w));
                } else {
                    *reinterpret_cast<float4*>(dst) = a;
                }
            }
        }
        if (p.mode != 1) {
            __syncthreads();

            // ---- stage 3: project.  acc rows = pixels, cols = output channels; this chunk's k slice ----
            // Few (pixel tile, channel tile) jobs and a long k: when there are fewer jobs than waves,
            // ksplit waves share a job, each reducing over a slice of the chunk's k.
            const int ksteps = kpc / KG, klen = (ksteps + p.ksplit - 1) / p.ksplit;
            auto partial = [&](int pt, int ot, int ks0, int ks1, f32x4 acc) {
                if constexpr (BF16) {
                    const bf16_t* ap = Ds + (pt * 16 + i) * p.ldd + 8 * g;
                    const bf16_t* bp = W2s + (ot * 16 + i) * p.ldw2 + 8 * g;
#pragma unroll 4
                    for (int ks = ks0; ks < ks1; ++ks)
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ld_bf16x8(ap + ks * 32), ld_bf16x8(bp + ks * 32), acc, 0, 0, 0);
                } else {
                    const float* ap = Ds + (pt * 16 + i) * p.ldd + g;
                    const float* bp = W2s + g * p.ldw2 + ot * 16 + i;
#pragma unroll 8
                    for (int ks = ks0; ks < ks1; ++ks)
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ap[ks * 4], bp[ks * 4 * p.ldw2], acc, 0, 0, 0);
                }
                return acc;
            };
            if (p.ksplit == 1) {
                if constexpr (CHUNKED) {
#pragma unroll
                    for (int jj = 0; jj < kInvresJobsPerWave; ++jj) {
                        const int job = wave + jj * kInvresWaves;
                        if (job < njobs) accj[jj] = partial(job % ptiles3, job / ptiles3, 0, ksteps, accj[jj]);
                    }
                } else {                               // one chunk: any number of jobs, stored as they finish
                    for (int job = wave; job < njobs; job += kInvresWaves)
                        emit(job % ptiles3, job / ptiles3,
                             partial(job % ptiles3, job / ptiles3, 0, ksteps, f32x4{0.f, 0.f, 0.f, 0.f}));
                }
            } else {                                   // njobs * ksplit <= number of waves
                const int job = wave / p.ksplit, kq = wave % p.ksplit;
                if (job < njobs)
                    accj[0] = partial(job % ptiles3, job / ptiles3, min(kq * klen, ksteps), min((kq + 1) * klen, ksteps), accj[0]);
            }
        }
        if (chunk + 1 < nchunks) __syncthreads();    // the next chunk overwrites the weights, E and D
    }
    if (p.mode == 1) return;

    // ---- epilogue: (sum the k split through LDS: the E region is free by now) + b2 (+ x), store ----
    if (p.ksplit == 1) {
        if constexpr (CHUNKED) {
#pragma unroll
            for (int jj = 0; jj < kInvresJobsPerWave; ++jj) {
                const int job = wave + jj * kInvresWaves;
                if (job < njobs) emit(job % ptiles3, job / ptiles3, accj[jj]);
            }
        }
    } else {
        float4* scratch = reinterpret_cast<float4*>(Es);
        if (wave / p.ksplit < njobs)
            scratch[wave * 64 + lane] = make_float4(accj[0][0], accj[0][1], accj[0][2], accj[0][3]);
        __syncthreads();
        if (wave < njobs) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            for (int q = 0; q < p.ksplit; ++q) {
                const float4 v = scratch[(wave * p.ksplit + q) * 64 + lane];
                acc[0] += v.x; acc[1] += v.y; acc[2] += v.z; acc[3] += v.w;
            }
            emit(wave % ptiles3, wave / ptiles3, acc);
        }
    }
}

// y = T( sum_s part[s] + b2 (+ x) ), slices added in index order; 4 consecutive channels per thread.
template <bool BF16>
__global__ __launch_bounds__(256) void invres_reduce_kernel(const float* __restrict__ part,
                                                            const float* __restrict__ b2, const void* __restrict__ xres,
                                                            void* __restrict__ y, long total, int Cout, int nsplit) {
    const long i4 = blockIdx.x * 256L + threadIdx.x;
    if (i4 * 4 >= total) return;
    float4 a = reinterpret_cast<const float4*>(part)[i4];
    for (int sp = 1; sp < nsplit; ++sp) {
        const float4 v = reinterpret_cast<const float4*>(part + (long)sp * total)[i4];
        a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
    }
    if (b2) {
        const float4 bv = *reinterpret_cast<const float4*>(b2 + (int)((i4 * 4) % Cout));
        a.x += bv.x; a.y += bv.y; a.z += bv.z; a.w += bv.w;
    }
    if constexpr (BF16) {
        if (xres) {
            const uint2 u = reinterpret_cast<const uint2*>(xres)[i4];
            a.x += lo_bf16(u.x); a.y += hi_bf16(u.x); a.z += lo_bf16(u.y); a.w += hi_bf16(u.y);
        }
        reinterpret_cast<uint2*>(y)[i4] = make_uint2(pack_bf16(a.x, a.y), pack_bf16(a.z, a.w));
    } else {
        if (xres) {
            const float4 u = reinterpret_cast<const float4*>(xres)[i4];
            a.x += u.x; a.y += u.y; a.z += u.z; a.w += u.w;
        }
        reinterpret_cast<float4*>(y)[i4] = a;
    }
}


constexpr size_t kInvresLdsMax = 160 * 1024;

// Lay out a tile with the fewest chunks of expanded channels that fit LDS (chunks balanced, widths
// multiples of 32).  Returns the byte count, or 0 when the tile cannot run: no chunk width fits, or it
// has more stage-3 jobs than the waves can hold accumulators for.
static size_t plan_tile(InvresParams& p, bool bf16, int stride, int toh, int tow, int ksize) {
    size_t smem = plan_layout(p, bf16, stride, toh, tow, ksize, p.Cexp);
    if (smem <= kInvresLdsMax) return smem;
    const int njobs = round_up(toh * tow, 16) / 16 * (round_up(p.Cout, 16) / 16);
    if (njobs > kInvresWaves * kInvresJobsPerWave) return 0;
    for (int cc = (p.Cexp - 1) / 32 * 32; cc >= 32; cc -= 32) {
        if (plan_layout(p, bf16, stride, toh, tow, ksize, cc) > kInvresLdsMax) continue;
        const int nch = (p.Cexp + cc - 1) / cc;
        const int bal = round_up((p.Cexp + nch - 1) / nch, 32);      // <= cc: same chunk count, balanced
        return plan_layout(p, bf16, stride, toh, tow, ksize, bal);
    }
    return 0;
}

// Cost of the channel split's reduction pass: a dependent launch, then its traffic at a few TB/s.
constexpr double kSplitReduceUs = 3.0, kSplitReduceBytesPerUs = 3.0e6;

// Predicted kernel time (microseconds) of a planned tile: a linear model of the work one workgroup
// does between its barriers, times the number of rounds the launch needs on the chip's 256 compute
// units.  In the paper's terms the tile size trades the re-computation of E's halo (and, here, the
// weights every workgroup stages for itself) against parallelism; where the paper tunes that trade
// by search, this model was fitted (non-negative least squares, relative error) to measured times of
// all candidate tiles over 21 block shapes on MI355X (mean error 5%; the tile it picks is within
// 3% of the best candidate on every one of them, also when that shape is left out of the fit).
//   units per workgroup: stage-1 jobs and matrix-instruction steps per wave, stage-2 iterations per
//   thread (and their taps), stage-3 steps per wave, KB of weights and of the X tile staged, chunks
//   channel split: every workgroup runs one chunk (its share of the weights), nsplit times as many
//   workgroups, plus the reduction pass (a dependent launch and (nsplit + 1) passes over the output)
static double predict_us(const InvresParams& p, bool bf16, int ksize, size_t smem) {
    constexpr int kCus = 256;
    const int kg = bf16 ? 32 : 4, es = bf16 ? 2 : 4;
    const bool split = p.nsplit > 1;
    const long wgs = (long)p.N * p.tiles_h * p.tiles_w * (split ? p.nsplit : 1);
    const int nch = split ? 1 : p.nchunks;
    const double cexp_wg = split ? (double)p.CC : (double)p.Cexp;      // expanded channels a workgroup stages
    auto cdiv = [](long a, long b) { return (a + b - 1) / b; };
    const double s1_jobs = p.mode == 2 ? 0.0 : (double)cdiv((long)(p.PEpad / 16) * (p.CC / 16), kInvresWaves) * nch;
    const double s1_steps = s1_jobs * (p.KP1 / kg);
    const double s2_it = (double)cdiv((long)p.TOH * p.TOW * (p.KPC / 4), kInvresThreads) * nch;
    const double s2_fma = s2_it * ksize * ksize;
    const int njobs = (p.POpad / 16) * (p.CoutP / 16), ksteps = p.KPC / kg;
    const double s3_steps = p.mode == 1 ? 0.0
                            : (njobs < kInvresWaves ? (double)cdiv(ksteps, p.ksplit) * nch
                                                    : (double)cdiv(njobs, kInvresWaves) * nch * ksteps);
    const double w_kb = ((p.mode == 2 ? 0.0 : (double)p.Cin * cexp_wg) + (p.mode == 1 ? 0.0 : cexp_wg * p.Cout) +
                         (double)ksize * ksize * cexp_wg) * es / 1024.0;
    const double x_kb = (double)p.PE * (p.mode == 2 ? cexp_wg : p.Cin) * es / 1024.0;
    const double t_wg = 2.156 + 2.198 * nch + 0.3036 * s1_jobs + 0.0417 * s1_steps + 0.3625 * s2_it +
                        0.0523 * s2_fma + 0.075 * s3_steps + 0.0089 * w_kb + 0.2013 * x_kb;
    // two workgroups share a compute unit when LDS and registers allow (single-chunk kernel, half the
    // LDS) and there are more workgroups than compute units; a shared unit runs each 1.5x slower
    const bool two = wgs > kCus && nch == 1 && smem <= kInvresLdsMax / 2;
    const double rounds = (double)cdiv(wgs, two ? 2 * kCus : kCus);
    double t = 1.208 + rounds * (two ? 1.5 : 1.0) * t_wg;
    if (split) t += kSplitReduceUs + (double)(p.nsplit + 1) * p.N * p.OH * p.OW * p.Cout * 4.0 / kSplitReduceBytesPerUs;
    return t;
}

// tile_cfg: -1 = built-in choice; otherwise tile candidate + 16 * channel-split option.
static const int kTileCand[][2] = {{2, 14}, {4, 4}, {1, 14}, {2, 2}, {4, 8}, {7, 7}, {2, 8}, {1, 8},
                                   {1, 2}, {2, 4}, {3, 3}, {1, 4}, {2, 3}, {1, 1}, {3, 4}, {2, 7}};
constexpr int kNumTiles = (int)(sizeof(kTileCand) / sizeof(kTileCand[0]));
// channel-split options: 0 = one workgroup per tile, else the widest chunk (expanded channels) a
// workgroup may take; the chunks are then balanced to multiples of 32
static const int kSplitCC[] = {0, 32, 64, 96, 128, 192, 256, 384};
constexpr int kNumSplits = (int)(sizeof(kSplitCC) / sizeof(kSplitCC[0]));
int fused_invres_num_cfgs() { return kNumTiles * kNumSplits; }

// Plan tile candidate `tile` with split option `so`.  Returns the LDS byte count, 0 when it cannot run
// (does not fit, or the option does not apply: no reduction to split, a single chunk anyway).
static size_t plan_candidate(InvresParams& p, bool bf16, int stride, int ksize, int tile, int so) {
    const int toh = kTileCand[tile][0], tow = kTileCand[tile][1];
    p.nsplit = 1;
    if (so == 0) return plan_tile(p, bf16, stride, toh, tow, ksize);
    if (p.mode == 1 || kSplitCC[so] >= p.Cexp) return 0;
    const int nch = (p.Cexp + kSplitCC[so] - 1) / kSplitCC[so];
    const int bal = round_up((p.Cexp + nch - 1) / nch, 32);          // <= the option's width
    const size_t smem = plan_layout(p, bf16, stride, toh, tow, ksize, bal);
    if (smem > kInvresLdsMax || p.nchunks < 2 || p.nchunks > 65535) return 0;
    p.nsplit = p.nchunks;
    return smem;
}

size_t invres_split_bytes(const InvresParams& p) {
    return p.nsplit > 1 ? (size_t)p.nsplit * p.N * p.OH * p.OW * p.Cout * sizeof(float) : 0;
}

// Fill p's tile fields for tile_cfg (-1: the candidate with the lowest predicted time among those whose
// partials fit ws_bytes of workspace).  Returns the LDS byte count, 0 when nothing fits; *chosen = the
// candidate's index, *us = its predicted time.
static size_t choose_tile(InvresParams& p, bool bf16, int stride, int ksize, int tile_cfg, size_t ws_bytes,
                          int* chosen, double* us) {
    int best = -1;
    double best_us = 0.0;
    if (tile_cfg >= 0 && tile_cfg < fused_invres_num_cfgs()) {
        best = tile_cfg;
    } else {
        for (int c = 0; c < fused_invres_num_cfgs(); ++c) {
            const size_t sz = plan_candidate(p, bf16, stride, ksize, c % kNumTiles, c / kNumTiles);
            if (sz == 0 || invres_split_bytes(p) > ws_bytes) continue;
            const double t = predict_us(p, bf16, ksize, sz);
            if (best < 0 || t < best_us) { best = c; best_us = t; }
        }
        if (best < 0) return 0;
    }
    const size_t smem = plan_candidate(p, bf16, stride, ksize, best % kNumTiles, best / kNumTiles);
    if (smem == 0 || invres_split_bytes(p) > ws_bytes) return 0;
    if (chosen) *chosen = best;
    if (us) *us = predict_us(p, bf16, ksize, smem);
    return smem;
}

// Host-only query of the plan a launch would use with ws_bytes of workspace (no GPU call).
// out: config, tile rows, tile columns, chunks per workgroup, chunk width, LDS bytes, workgroups per tile
int fused_invres_plan(int N, int H, int W, int Cin, int Cexp, int Cout, int stride, int ksize, bool bf16,
                      int tile_cfg, int mode, size_t ws_bytes, int out[7], float* predicted_us) {
    if ((ksize != 3 && ksize != 5) || (stride != 1 && stride != 2)) return -1;
    InvresParams p = {};
    p.mode = mode;
    p.N = N; p.H = H; p.W = W; p.Cin = Cin; p.Cexp = Cexp; p.Cout = Cout;
    p.OH = (H - 1) / stride + 1; p.OW = (W - 1) / stride + 1;
    int chosen = -1;
    double us = 0.0;
    const size_t smem = choose_tile(p, bf16, stride, ksize, tile_cfg, ws_bytes, &chosen, &us);
    if (smem == 0) return -1;
    out[0] = chosen; out[1] = p.TOH; out[2] = p.TOW; out[3] = p.nsplit > 1 ? 1 : p.nchunks; out[4] = p.CC;
    out[5] = (int)smem; out[6] = p.nsplit;
    // a shape of the specialisation table runs the specialised instantiation: measured at 0.6 x (one workgroup
    // per tile) and 0.8 x (channel split: the reduction pass is unchanged) the general instantiation's time
    if (tile_cfg < 0 && ksize == 3) {
        for (int id = 1; id < kNumInvresSpecs; ++id) {
            if ((kInvresSpecs[id].bf16 != 0) != bf16 || kInvresSpecs[id].stride != stride) continue;
            p.residual = kInvresSpecs[id].residual;
            if (invres_matches_spec(p, id)) { us *= p.nsplit > 1 ? 0.8 : 0.6; break; }
        }
    }
    if (predicted_us) *predicted_us = (float)us;
    return 0;
}

// Workspace the preferred plan needs (0 when it does not split the expanded channels).
size_t fused_invres_workspace(int N, int H, int W, int Cin, int Cexp, int Cout, int stride, int ksize, bool bf16,
                              int tile_cfg, int mode) {
    if ((ksize != 3 && ksize != 5) || (stride != 1 && stride != 2)) return 0;
    InvresParams p = {};
    p.mode = mode;
    p.N = N; p.H = H; p.W = W; p.Cin = Cin; p.Cexp = Cexp; p.Cout = Cout;
    p.OH = (H - 1) / stride + 1; p.OW = (W - 1) / stride + 1;
    if (choose_tile(p, bf16, stride, ksize, tile_cfg, ~(size_t)0, nullptr, nullptr) == 0) return 0;
    return invres_split_bytes(p);
}

// Launch the shape-specialised instantiation whose geometry equals the run-time plan, if there is one.
template <int ID>
static bool try_invres_spec(const InvresParams& p, bool bf16, int stride, int residual, dim3 grid, size_t smem, hipStream_t s,
                            hipError_t* err) {
    constexpr InvresSpecShape q = kInvresSpecs[ID];
    if (bf16 != (q.bf16 != 0) || stride != q.stride || residual != q.residual || !invres_matches_spec(p, ID)) return false;
    constexpr size_t kLdsMax = 160 * 1024;
    auto kern = fused_invres_kernel<(q.bf16 != 0), q.stride, 3, false, (q.split != 0), ID>;
    *err = allow_dynamic_lds<fused_invres_kernel<(q.bf16 != 0), q.stride, 3, false, (q.split != 0), ID>>((int)kLdsMax);
    if (*err != hipSuccess) return true;
    prof_start(0, s);
    prof_shape(0, grid.x * grid.y, kInvresThreads);
    hipLaunchKernelGGL(kern, grid, dim3(kInvresThreads), smem, s, p);
    return true;
}
template <int... IDS>
static bool launch_invres_spec(const InvresParams& p, bool bf16, int stride, int residual, dim3 grid, size_t smem, hipStream_t s,
                               std::integer_sequence<int, IDS...>, hipError_t* err) {
    return (try_invres_spec<IDS + 1>(p, bf16, stride, residual, grid, smem, s, err) || ...);
}

hipError_t fused_invres(const void* x, const void* w1, const float* b1, const void* wd, const float* bd,
                        const void* w2, const float* b2, void* y, int N, int H, int W, int Cin,
                        int Cexp, int Cout, int stride, int residual, bool bf16, int tile_cfg,
                        hipStream_t s, int mode, int ksize, void* workspace, size_t ws_bytes) {
    if (ksize != 3 && ksize != 5) return hipErrorInvalidValue;
    // The plan (tile, chunking, split, LDS layout) depends on the shape only; walking all candidates costs
    // as much host time as the kernel runs on the small blocks, so the last few plans are kept per thread.
    struct PlanKey {
        int v[11];
        size_t ws;
    };
    struct PlanSlot {
        PlanKey key;
        InvresParams p;
        size_t smem;
        bool valid;
    };
    static thread_local PlanSlot plans[8] = {};
    static thread_local int next_slot = 0;
    const PlanKey key = {{N, H, W, Cin, Cexp, Cout, stride, ksize, bf16 ? 1 : 0, tile_cfg, mode}, workspace ? ws_bytes : 0};
    const PlanSlot* hit = nullptr;
    for (const PlanSlot& sl : plans) {
        if (!sl.valid || sl.key.ws != key.ws) continue;
        bool same = true;
        for (int q = 0; q < 11; ++q) same = same && sl.key.v[q] == key.v[q];
        if (same) { hit = &sl; break; }
    }
    InvresParams p;
    size_t smem;
    if (hit) {
        p = hit->p;
        smem = hit->smem;
    } else {
        p = InvresParams{};
        p.mode = mode;
        p.N = N; p.H = H; p.W = W; p.Cin = Cin; p.Cexp = Cexp; p.Cout = Cout;
        p.OH = (H - 1) / stride + 1; p.OW = (W - 1) / stride + 1;
        p.nsplit = 1;
        smem = choose_tile(p, bf16, stride, ksize, tile_cfg, key.ws, nullptr, nullptr);
        if (smem == 0) return hipErrorInvalidValue;
        PlanSlot& sl = plans[next_slot];
        next_slot = (next_slot + 1) % 8;
        sl.key = key; sl.p = p; sl.smem = smem; sl.valid = true;
    }
    p.x = x; p.w1 = w1; p.b1 = b1; p.wd = wd; p.bd = bd; p.w2 = w2; p.b2 = b2; p.y = y;
    p.residual = residual;
    p.part = static_cast<float*>(workspace);
    constexpr size_t kLdsMax = kInvresLdsMax;
    const bool split = p.nsplit > 1;
    const dim3 grid((unsigned)(N * p.tiles_h * p.tiles_w), (unsigned)p.nsplit);
#define AGO_LAUNCH_INVRES_KC(BF, ST, KS, CH, SP)                                                        \
    do {                                                                                                \
        auto kern = fused_invres_kernel<BF, ST, KS, CH, SP>;                                            \
        if (hipError_t e = allow_dynamic_lds<fused_invres_kernel<BF, ST, KS, CH, SP>>((int)kLdsMax); e != hipSuccess) return e; \
        prof_start(0, s);                                                                               \
        prof_shape(0, grid.x * grid.y, kInvresThreads);                                                 \
        hipLaunchKernelGGL(kern, grid, dim3(kInvresThreads), smem, s, p);                               \
    } while (0)
#define AGO_LAUNCH_INVRES_K(BF, ST, KS)                                                                 \
    do {                                                                                                \
        if (split) AGO_LAUNCH_INVRES_KC(BF, ST, KS, false, true);                                       \
        else if (p.nchunks == 1) AGO_LAUNCH_INVRES_KC(BF, ST, KS, false, false);                        \
        else AGO_LAUNCH_INVRES_KC(BF, ST, KS, true, false);                                             \
    } while (0)
#define AGO_LAUNCH_INVRES(BF, ST)                                                                       \
    do {                                                                                                \
        if (ksize == 3) AGO_LAUNCH_INVRES_K(BF, ST, 3); else AGO_LAUNCH_INVRES_K(BF, ST, 5);            \
    } while (0)
    bool launched = false;
    if (ksize == 3 && tile_cfg < 0) {
        hipError_t spec_err = hipSuccess;
        launched = launch_invres_spec(p, bf16, stride, residual, grid, smem, s, std::make_integer_sequence<int, kNumInvresSpecs - 1>{}, &spec_err);
        if (spec_err != hipSuccess) return spec_err;
    }
    if (launched) {}
    else if (bf16) { if (stride == 1) AGO_LAUNCH_INVRES(true, 1); else AGO_LAUNCH_INVRES(true, 2); }
    else { if (stride == 1) AGO_LAUNCH_INVRES(false, 1); else AGO_LAUNCH_INVRES(false, 2); }
#undef AGO_LAUNCH_INVRES
#undef AGO_LAUNCH_INVRES_K
#undef AGO_LAUNCH_INVRES_KC
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !split) {
        prof_stop(0, s);
        return e;
    }
    // sum the partial projections; b2 and the residual were left to this pass
    const long total = (long)N * p.OH * p.OW * Cout;
    const unsigned rgrid = (unsigned)((total / 4 + 255) / 256);
    if (bf16)
        hipLaunchKernelGGL(invres_reduce_kernel<true>, dim3(rgrid), dim3(256), 0, s, p.part, b2, residual ? x : nullptr, y,
                           total, Cout, p.nsplit);
    else
        hipLaunchKernelGGL(invres_reduce_kernel<false>, dim3(rgrid), dim3(256), 0, s, p.part, b2, residual ? x : nullptr, y,
                           total, Cout, p.nsplit);
    prof_stop(0, s);      // the event pair brackets the whole entry point, the reduction included
    return hipGetLastError();
}

}  // namespace ago
