// C ABI entry points: validate on the host (no HIP call before validation passes), then launch.
#include <hip/hip_runtime.h>
#include <mutex>
#include <vector>
#include "ago_host.hpp"
#include "ago_launch.hpp"
#include "ago_dev.hpp"

using namespace ago;

static inline ago_status from_hip(hipError_t e) {
    if (e == hipSuccess) return AGO_OK;
    return e == hipErrorInvalidValue ? AGO_ERR_UNSUPPORTED : AGO_ERR_LAUNCH;
}
static inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
static inline size_t esize(ago_dtype dt) { return dt == AGO_BF16 ? 2 : 4; }

// ---------------------------------------------------------------- instrumentation
namespace {
struct ProfRing {
    std::vector<hipEvent_t> start, mid, stop;      // mid: after the entry point's first kernel, when it launches two
    std::vector<char> has_mid;
    long calls = 0;
};
ProfRing g_prof[4];
int g_prof_cap = 0;
unsigned g_prof_mask = 0xFu;      // bit op: that fused entry point records events
unsigned g_last_grid[4] = {0, 0, 0, 0}, g_last_block[4] = {0, 0, 0, 0};
__global__ void empty_kernel() {}

// Matrix-instruction-only loops: what the matrix cores sustain with every operand in registers.
// bf16: six independent 32x32x16 accumulators per wave; fp32: six 32x32x2.
template <bool BF16>
__global__ __launch_bounds__(512) void mfma_only_kernel(float* out, int iters) {
    ago::f32x16 acc[6];
#pragma unroll
    for (int j = 0; j < 6; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
    ago::bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = (ago::bf16_t)(float)(threadIdx.x & 3); b[e] = (ago::bf16_t)(float)(e & 1); }
    const float af = (float)(threadIdx.x & 3), bf = 0.5f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 6; ++j) {
            if constexpr (BF16) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
            else acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af, bf, acc[j], 0, 0, 0);
        }
    }
    float sum = 0.0f;
#pragma unroll
    for (int j = 0; j < 6; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += acc[j][r];
    out[blockIdx.x * blockDim.x + threadIdx.x] = sum;
}
}  // namespace

namespace ago {
void prof_start(int op, hipStream_t s) {
    if (g_prof_cap > 0 && ((g_prof_mask >> op) & 1u)) {
        const long i = g_prof[op].calls % g_prof_cap;
        g_prof[op].has_mid[i] = 0;
        (void)hipEventRecord(g_prof[op].start[i], s);
    }
}
void prof_mid(int op, hipStream_t s) {
    if (g_prof_cap > 0 && ((g_prof_mask >> op) & 1u)) {
        const long i = g_prof[op].calls % g_prof_cap;
        (void)hipEventRecord(g_prof[op].mid[i], s);
        g_prof[op].has_mid[i] = 1;
    }
}
void prof_stop(int op, hipStream_t s) {
    if (g_prof_cap > 0 && ((g_prof_mask >> op) & 1u)) {
        (void)hipEventRecord(g_prof[op].stop[g_prof[op].calls % g_prof_cap], s);
        ++g_prof[op].calls;
    }
}
void prof_shape(int op, unsigned grid, unsigned block) { g_last_grid[op] = grid; g_last_block[op] = block; }
}  // namespace ago

// ---------------------------------------------------------------- scratch owned by the library
// ago_fused_invres_noalloc keeps its cross-workgroup partial sums here instead of in a caller workspace.
// Every GPU the library runs on holds its own copy of the array until the process ends.  In host code the
// array's name is only a stand-in: the device address comes from hipGetSymbolAddress, once per device.
namespace {
static __device__ __align__(256) unsigned char scratch[AGO_NOALLOC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

hipError_t scratch_address(void** out) {
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)); e != hipSuccess) return e;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace

extern "C" {

int ago_profile_last_launch(ago_op op, int* grid, int* block) {
    if ((int)op < 0 || (int)op > 3 || !grid || !block || g_last_block[(int)op] == 0) return -1;
    *grid = (int)g_last_grid[(int)op]; *block = (int)g_last_block[(int)op];
    return 0;
}

int ago_bench_empty_kernel(int grid, int block, void* hip_stream) {
    if (grid <= 0 || block <= 0 || block > 1024) return -1;
    hipLaunchKernelGGL(empty_kernel, dim3((unsigned)grid), dim3((unsigned)block), 0, reinterpret_cast<hipStream_t>(hip_stream));
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int ago_profile_enable(int capacity) {
    for (auto& r : g_prof) {
        for (hipEvent_t e : r.start) (void)hipEventDestroy(e);
        for (hipEvent_t e : r.mid) (void)hipEventDestroy(e);
        for (hipEvent_t e : r.stop) (void)hipEventDestroy(e);
        r.start.clear(); r.mid.clear(); r.stop.clear(); r.has_mid.clear(); r.calls = 0;
    }
    g_prof_cap = 0;
    if (capacity <= 0) return 0;
    if (capacity > 4096) return -1;
    for (auto& r : g_prof) {
        r.start.resize(capacity); r.mid.resize(capacity); r.stop.resize(capacity); r.has_mid.assign(capacity, 0);
        for (int i = 0; i < capacity; ++i)
            if (hipEventCreate(&r.start[i]) != hipSuccess || hipEventCreate(&r.mid[i]) != hipSuccess ||
                hipEventCreate(&r.stop[i]) != hipSuccess) return -1;
    }
    g_prof_cap = capacity;
    return 0;
}

int ago_profile_select(unsigned op_mask) {
    if (op_mask & ~0xFu) return -1;
    g_prof_mask = op_mask;
    return 0;
}

int ago_profile_read_split(ago_op op, float* total_ms, float* first_kernel_ms, int* count) {
    if ((int)op < 0 || (int)op > 3 || !total_ms || !count || g_prof_cap <= 0) return -1;
    ProfRing& r = g_prof[(int)op];
    const int n = (int)(r.calls < g_prof_cap ? r.calls : g_prof_cap);
    float tot = 0.f, first = 0.f;
    for (int i = 0; i < n; ++i) {
        float ms = 0.f, ms1 = 0.f;
        if (hipEventSynchronize(r.stop[i]) != hipSuccess) return -1;
        if (hipEventElapsedTime(&ms, r.start[i], r.stop[i]) != hipSuccess) return -1;
        if (r.has_mid[i]) {
            if (hipEventElapsedTime(&ms1, r.start[i], r.mid[i]) != hipSuccess) return -1;
        } else {
            ms1 = ms;
        }
        tot += ms;
        first += ms1;
    }
    *total_ms = tot; *count = n;
    if (first_kernel_ms) *first_kernel_ms = first;
    r.calls = 0;
    return 0;
}

int ago_profile_read(ago_op op, float* total_ms, int* count) {
    return ago_profile_read_split(op, total_ms, nullptr, count);
}

int ago_bench_mfma_kernel(ago_dtype dt, int iters, void* out, size_t out_bytes, double* flops, void* hip_stream) {
    if (!out || iters <= 0 || (dt != AGO_BF16 && dt != AGO_F32)) return -1;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return -1;
    const unsigned grid = (unsigned)prop.multiProcessorCount, block = 512;
    if (out_bytes < (size_t)grid * block * sizeof(float)) return -1;
    hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
    if (dt == AGO_BF16) hipLaunchKernelGGL(mfma_only_kernel<true>, dim3(grid), dim3(block), 0, s, (float*)out, iters);
    else hipLaunchKernelGGL(mfma_only_kernel<false>, dim3(grid), dim3(block), 0, s, (float*)out, iters);
    if (flops) *flops = (double)grid * (block / 64) * iters * 6.0 * (dt == AGO_BF16 ? 32768.0 : 4096.0);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

float ago_profile_event_overhead_ms(void* hip_stream, int pairs) {
    if (pairs <= 0 || pairs > 1024) return -1.0f;
    hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
    std::vector<hipEvent_t> a(pairs), b(pairs);
    for (int i = 0; i < pairs; ++i)
        if (hipEventCreate(&a[i]) != hipSuccess || hipEventCreate(&b[i]) != hipSuccess) return -1.0f;
    for (int i = 0; i < pairs; ++i) {
        (void)hipEventRecord(a[i], s);
        (void)hipEventRecord(b[i], s);
    }
    float tot = 0.f;
    bool ok = true;
    for (int i = 0; i < pairs; ++i) {
        float ms = 0.f;
        ok = ok && hipEventSynchronize(b[i]) == hipSuccess && hipEventElapsedTime(&ms, a[i], b[i]) == hipSuccess;
        tot += ms;
    }
    for (int i = 0; i < pairs; ++i) { (void)hipEventDestroy(a[i]); (void)hipEventDestroy(b[i]); }
    return ok ? tot / pairs : -1.0f;
}

// ---------------------------------------------------------------- fused subgraphs
ago_status ago_fused_invres(const void* x, const void* w1, const float* b1, const void* wd,
                            const float* bd, const void* w2, const float* b2, void* y, int N, int H,
                            int W, int Cin, int Cexp, int Cout, int stride, int residual, ago_dtype dt,
                            void* workspace, size_t workspace_bytes, void* hip_stream) {
    ago_status st = check_invres(x, w1, wd, w2, y, b1, bd, b2, N, H, W, Cin, Cexp, Cout, stride, residual, dt);
    if (st != AGO_OK) return st;
    if (workspace && reinterpret_cast<uintptr_t>(workspace) % 16) return AGO_ERR_ALIGN;
    return from_hip(fused_invres(x, w1, b1, wd, bd, w2, b2, y, N, H, W, Cin, Cexp, Cout, stride,
                                 residual, dt == AGO_BF16, tile_config(AGO_OP_FUSED_INVRES),
                                 as_stream(hip_stream), 0, 3, workspace, workspace_bytes));
}

ago_status ago_fused_invres_k(const void* x, const void* w1, const float* b1, const void* wd,
                              const float* bd, const void* w2, const float* b2, void* y, int N, int H,
                              int W, int Cin, int Cexp, int Cout, int stride, int ksize, int residual,
                              ago_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream) {
    ago_status st = check_invres(x, w1, wd, w2, y, b1, bd, b2, N, H, W, Cin, Cexp, Cout, stride, residual, dt);
    if (st != AGO_OK) return st;
    if (ksize != 3 && ksize != 5) return AGO_ERR_UNSUPPORTED;
    if (workspace && reinterpret_cast<uintptr_t>(workspace) % 16) return AGO_ERR_ALIGN;
    return from_hip(fused_invres(x, w1, b1, wd, bd, w2, b2, y, N, H, W, Cin, Cexp, Cout, stride,
                                 residual, dt == AGO_BF16, tile_config(AGO_OP_FUSED_INVRES),
                                 as_stream(hip_stream), 0, ksize, workspace, workspace_bytes));
}

ago_status ago_fused_invres_noalloc(const void* x, const void* w1, const float* b1, const void* wd,
                                    const float* bd, const void* w2, const float* b2, void* y, int N, int H,
                                    int W, int Cin, int Cexp, int Cout, int stride, int ksize, int residual,
                                    ago_dtype dt, void* hip_stream) {
    ago_status st = check_invres(x, w1, wd, w2, y, b1, bd, b2, N, H, W, Cin, Cexp, Cout, stride, residual, dt);
    if (st != AGO_OK) return st;
    if (ksize != 3 && ksize != 5) return AGO_ERR_UNSUPPORTED;
    const int dims[8] = {N, H, W, Cin, Cexp, Cout, stride, ksize};
    if (ago::workspace_bytes(AGO_OP_FUSED_INVRES, dims, 8, dt) > AGO_NOALLOC_SCRATCH_BYTES) return AGO_ERR_WORKSPACE;
    void* ptr = nullptr;
    if (hipError_t e = scratch_address(&ptr); e != hipSuccess) return from_hip(e);
    return from_hip(fused_invres(x, w1, b1, wd, bd, w2, b2, y, N, H, W, Cin, Cexp, Cout, stride,
                                 residual, dt == AGO_BF16, tile_config(AGO_OP_FUSED_INVRES),
                                 as_stream(hip_stream), 0, ksize, ptr, AGO_NOALLOC_SCRATCH_BYTES));
}

ago_status ago_fused_invres_plan(int N, int H, int W, int Cin, int Cexp, int Cout, int stride, int ksize,
                                 ago_dtype dt, size_t workspace_bytes, int plan[7], float* predicted_us) {
    if (!plan) return AGO_ERR_NULL;
    if (dt != AGO_F32 && dt != AGO_BF16) return AGO_ERR_DTYPE;
    if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cexp <= 0 || Cout <= 0) return AGO_ERR_SHAPE;
    if (stride != 1 && stride != 2) return AGO_ERR_SHAPE;
    if (Cin % 8 || Cexp % 16 || Cout % 8 || (ksize != 3 && ksize != 5)) return AGO_ERR_UNSUPPORTED;
    return fused_invres_plan(N, H, W, Cin, Cexp, Cout, stride, ksize, dt == AGO_BF16,
                             tile_config(AGO_OP_FUSED_INVRES), 0, workspace_bytes, plan, predicted_us) == 0
               ? AGO_OK : AGO_ERR_UNSUPPORTED;
}

ago_status ago_fused_pw_dw_k(const void* x, const void* w1, const float* b1, const void* wd, const float* bd,
                             void* y, int N, int H, int W, int Cin, int Cexp, int stride, int ksize, ago_dtype dt,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
    (void)workspace; (void)workspace_bytes;
    ago_status st = check_pw_dw(x, w1, wd, y, b1, bd, N, H, W, Cin, Cexp, stride, dt);
    if (st != AGO_OK) return st;
    if (ksize != 3 && ksize != 5) return AGO_ERR_UNSUPPORTED;
    return from_hip(fused_invres(x, w1, b1, wd, bd, nullptr, nullptr, y, N, H, W, Cin, Cexp, 16, stride, 0,
                                 dt == AGO_BF16, tile_config(AGO_OP_FUSED_INVRES), as_stream(hip_stream), 1, ksize));
}

ago_status ago_fused_pw_dw(const void* x, const void* w1, const float* b1, const void* wd, const float* bd,
                           void* y, int N, int H, int W, int Cin, int Cexp, int stride, ago_dtype dt,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
    return ago_fused_pw_dw_k(x, w1, b1, wd, bd, y, N, H, W, Cin, Cexp, stride, 3, dt, workspace, workspace_bytes,
                             hip_stream);
}

ago_status ago_fused_dw_pw_k(const void* x, const void* wd, const float* bd, const void* w2, const float* b2,
                             void* y, int N, int H, int W, int C, int Cout, int stride, int ksize, ago_dtype dt,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
    ago_status st = check_dw_pw(x, wd, w2, y, bd, b2, N, H, W, C, Cout, stride, dt);
    if (st != AGO_OK) return st;
    if (ksize != 3 && ksize != 5) return AGO_ERR_UNSUPPORTED;
    if (workspace && reinterpret_cast<uintptr_t>(workspace) % 16) return AGO_ERR_ALIGN;
    return from_hip(fused_invres(x, nullptr, nullptr, wd, bd, w2, b2, y, N, H, W, 8, C, Cout, stride, 0,
                                 dt == AGO_BF16, tile_config(AGO_OP_FUSED_INVRES), as_stream(hip_stream), 2, ksize,
                                 workspace, workspace_bytes));
}

ago_status ago_fused_dw_pw(const void* x, const void* wd, const float* bd, const void* w2, const float* b2,
                           void* y, int N, int H, int W, int C, int Cout, int stride, ago_dtype dt,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
    return ago_fused_dw_pw_k(x, wd, bd, w2, b2, y, N, H, W, C, Cout, stride, 3, dt, workspace, workspace_bytes,
                             hip_stream);
}

ago_status ago_fused_dw_dw(const void* x, const void* wa, const float* ba, const void* wb, const float* bb,
                           void* y, int N, int H, int W, int C, int stride, ago_dtype dt,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
    (void)workspace; (void)workspace_bytes;
    const void* ps[6] = {x, wa, wb, y, ba, bb};
    ago_status st = check_ptrs(ps, 4, 6);
    if (st != AGO_OK) return st;
    if (!valid_dtype(dt)) return AGO_ERR_DTYPE;
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || (stride != 1 && stride != 2)) return AGO_ERR_SHAPE;
    if (C % 4 || !fits31(N, H, W, C)) return AGO_ERR_UNSUPPORTED;
    return from_hip(fused_dw_dw(x, wa, ba, wb, bb, y, N, H, W, C, stride, dt == AGO_BF16, as_stream(hip_stream)));
}

ago_status ago_fused_pw_pw(const void* x, const void* w1, const float* b1, const void* w2, const float* b2,
                           void* y, int N, int H, int W, int Cin, int Cmid, int Cout, ago_act act,
                           ago_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (N <= 0 || H <= 0 || W <= 0) return x && w1 && w2 && y ? AGO_ERR_SHAPE : AGO_ERR_NULL;
    const long long m = (long long)N * H * W;
    if (m >= (1LL << 31)) return AGO_ERR_UNSUPPORTED;
    return ago_fused_ffn(x, w1, b1, w2, b2, y, (int)m, Cin, Cmid, Cout, act, dt, workspace, workspace_bytes,
                         hip_stream);
}

ago_status ago_fused_conv_chain(const void* x, const void* wa, const float* ba, const void* wb,
                                const float* bb, void* y, int N, int H, int W, int C, int residual,
                                ago_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream) {
    (void)workspace; (void)workspace_bytes;
    ago_status st = check_conv_chain(x, wa, wb, y, ba, bb, N, H, W, C, dt);
    if (st != AGO_OK) return st;
    return from_hip(fused_conv_chain(x, wa, ba, wb, bb, y, N, H, W, residual,
                                     tile_config(AGO_OP_FUSED_CONV_CHAIN), as_stream(hip_stream)));
}

ago_status ago_fused_ffn(const void* x, const void* w1, const float* b1, const void* w2,
                         const float* b2, void* y, int M, int K, int F, int K2, ago_act act,
                         ago_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream) {
    ago_status st = check_ffn(x, w1, w2, y, b1, b2, M, K, F, K2, act, dt);
    if (st != AGO_OK) return st;
    const int cfg = tile_config(AGO_OP_FUSED_FFN);
    const int picked = fused_ffn_pick_cfg(M, K, F, K2, cfg);
    if (picked < 0) return AGO_ERR_UNSUPPORTED;
    if ((long long)fused_ffn_nsplit(picked, F) * M * K2 >= (1LL << 31)) return AGO_ERR_UNSUPPORTED;  // 32-bit offsets
    const int dims[4] = {M, K, F, K2};
    st = check_workspace(workspace, workspace_bytes, ago::workspace_bytes(AGO_OP_FUSED_FFN, dims, 4, dt));
    if (st != AGO_OK) return st;
    return from_hip(fused_ffn(x, w1, b1, w2, b2, y, M, K, F, K2, act, cfg, workspace, as_stream(hip_stream)));
}

size_t ago_packed_weight_bytes(int K, int N) {
    return (K > 0 && N > 0 && K % 32 == 0 && N % 16 == 0) ? (size_t)K * (size_t)N * 2 : 0;
}

ago_status ago_pack_weight(const void* w, void* wp, int K, int N, ago_dtype dt, void* hip_stream) {
    ago_status st = check_pack_weight(w, wp, K, N, dt);
    if (st != AGO_OK) return st;
    return from_hip(pack_weight(w, wp, K, N, as_stream(hip_stream)));
}

int ago_gemm_packed_supported(int M, int K, int N) {
    return (M > 0 && K > 0 && N > 0 && gemm_packed_variant(M, K, N) != 0) ? 1 : 0;
}

ago_status ago_gemm_packed(const void* a, const void* wp, const float* bias, void* c, int M, int K, int N,
                           ago_act act, ago_dtype dt, void* hip_stream) {
    ago_status st = check_gemm_packed(a, wp, c, bias, M, K, N, act, dt);
    if (st != AGO_OK) return st;
    return from_hip(gemm_packed(a, wp, bias, c, M, K, N, act, as_stream(hip_stream)));
}

ago_status ago_unfused_ffn_packed(const void* x, const void* w1p, const float* b1, const void* w2p,
                                  const float* b2, void* y, int M, int K, int F, int K2, ago_act act,
                                  ago_dtype dt, void* workspace, size_t workspace_bytes, void* s) {
    if (!x || !w1p || !w2p || !y) return AGO_ERR_NULL;
    if (M <= 0 || K <= 0 || F <= 0 || K2 <= 0) return AGO_ERR_SHAPE;
    const int dims[4] = {M, K, F, K2};
    ago_status st = check_workspace(workspace, workspace_bytes, ago::workspace_bytes(AGO_OP_UNFUSED_FFN, dims, 4, dt));
    if (st != AGO_OK) return st;
    if (workspace_bytes == 0 || !workspace) return AGO_ERR_WORKSPACE;
    // both products are checked before the first is launched
    if (gemm_packed_variant(M, K, F) == 0 || gemm_packed_variant(M, F, K2) == 0) return AGO_ERR_UNSUPPORTED;
    st = ago_gemm_packed(x, w1p, b1, workspace, M, K, F, act, dt, s);
    if (st != AGO_OK) return st;
    return ago_gemm_packed(workspace, w2p, b2, y, M, F, K2, AGO_ACT_NONE, dt, s);
}

ago_status ago_fused_ffn_packed(const void* x, const void* w1p, const float* b1, const void* w2p,
                                const float* b2, void* y, int M, int K, int F, int K2, ago_act act,
                                ago_dtype dt, void* workspace, size_t workspace_bytes, void* hip_stream) {
    ago_status st = check_ffn_packed(x, w1p, w2p, y, b1, b2, M, K, F, K2, act, dt);
    if (st != AGO_OK) return st;
    const int dims[4] = {M, K, F, K2};
    st = check_workspace(workspace, workspace_bytes, ago::workspace_bytes(AGO_OP_FUSED_FFN_PACKED, dims, 4, dt));
    if (st != AGO_OK) return st;
    return from_hip(fused_ffn_packed(x, w1p, b1, w2p, b2, y, M, K, F, K2, act, workspace, as_stream(hip_stream)));
}

ago_status ago_fused_attn(const void* q, const void* k, const void* v, void* o, int B, int Hh, int S,
                          int D, float scale, ago_dtype dt, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
    (void)workspace; (void)workspace_bytes;
    ago_status st = check_attn(q, k, v, o, B, Hh, S, D, scale, dt);
    if (st != AGO_OK) return st;
    return from_hip(fused_attn(q, k, v, o, B, Hh, S, scale, tile_config(AGO_OP_FUSED_ATTN), as_stream(hip_stream),
                               0, 0, 0, D));
}

// ---------------------------------------------------------------- un-fused operators
ago_status ago_gemm(const void* a, const void* b, const float* bias, const void* res, void* c, int M,
                    int K, int N, ago_act act, ago_dtype dt, void* hip_stream) {
    const void* ps[5] = {a, b, c, bias, res};
    ago_status st = check_ptrs(ps, 3, 5);
    if (st != AGO_OK) return st;
    if (!valid_dtype(dt) || !valid_act(act)) return AGO_ERR_DTYPE;
    if (M <= 0 || K <= 0 || N <= 0) return AGO_ERR_SHAPE;
    if (K % 8 || N % 8 || !fits31(M, K > N ? K : N, 1, 1) || !fits31(K, N, 1, 1)) return AGO_ERR_UNSUPPORTED;
    return from_hip(dt == AGO_BF16 ? gemm_bf16(a, b, bias, res, c, M, K, N, act, as_stream(hip_stream))
                                   : gemm_f32(a, b, bias, res, c, M, K, N, act, as_stream(hip_stream)));
}

ago_status ago_conv1x1(const void* x, const void* w, const float* bias, const void* res, void* y, int N,
                       int H, int W, int Cin, int Cout, ago_act act, ago_dtype dt, void* hip_stream) {
    if (N <= 0 || H <= 0 || W <= 0) return (x && w && y) ? AGO_ERR_SHAPE : AGO_ERR_NULL;
    const long P = (long)N * H * W;
    if (P > 0x7fffffffL) return AGO_ERR_UNSUPPORTED;
    return ago_gemm(x, w, bias, res, y, (int)P, Cin, Cout, act, dt, hip_stream);
}

ago_status ago_dwconv3x3(const void* x, const void* w, const float* bias, void* y, int N, int H, int W,
                         int C, int stride, ago_act act, ago_dtype dt, void* hip_stream) {
    const void* ps[4] = {x, w, y, bias};
    ago_status st = check_ptrs(ps, 3, 4);
    if (st != AGO_OK) return st;
    if (!valid_dtype(dt) || !valid_act(act)) return AGO_ERR_DTYPE;
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || (stride != 1 && stride != 2)) return AGO_ERR_SHAPE;
    if (C % 8 || !fits31(N, H, W, C)) return AGO_ERR_UNSUPPORTED;
    return from_hip(dwconv3x3(x, w, bias, y, N, H, W, C, stride, act, dt == AGO_BF16, as_stream(hip_stream)));
}

ago_status ago_conv3x3(const void* x, const void* w, const float* bias, const void* res, void* y, int N,
                       int H, int W, int Cin, int Cout, ago_act act, ago_dtype dt, void* hip_stream) {
    const void* ps[5] = {x, w, y, bias, res};
    ago_status st = check_ptrs(ps, 3, 5);
    if (st != AGO_OK) return st;
    if (!valid_dtype(dt) || !valid_act(act)) return AGO_ERR_DTYPE;
    if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0) return AGO_ERR_SHAPE;
    if (dt != AGO_BF16 || Cin != 64 || Cout != 64 || !fits31(N, H, W, 64)) return AGO_ERR_UNSUPPORTED;
    return from_hip(conv3x3_bf16(x, w, bias, res, y, N, H, W, act, as_stream(hip_stream)));
}

ago_status ago_bias_act(const void* x, const float* bias, void* y, long P, int C, ago_act act,
                        ago_dtype dt, void* hip_stream) {
    const void* ps[3] = {x, y, bias};
    ago_status st = check_ptrs(ps, 2, 3);
    if (st != AGO_OK) return st;
    if (!valid_dtype(dt) || !valid_act(act)) return AGO_ERR_DTYPE;
    if (P <= 0 || C <= 0) return AGO_ERR_SHAPE;
    if (C % 8) return AGO_ERR_UNSUPPORTED;
    return from_hip(bias_act(x, bias, y, P, C, act, dt == AGO_BF16, as_stream(hip_stream)));
}

ago_status ago_add_act(const void* a, const void* b, void* y, long n, ago_act act, ago_dtype dt,
                       void* hip_stream) {
    const void* ps[3] = {a, b, y};
    ago_status st = check_ptrs(ps, 3, 3);
    if (st != AGO_OK) return st;
    if (!valid_dtype(dt) || !valid_act(act)) return AGO_ERR_DTYPE;
    if (n <= 0) return AGO_ERR_SHAPE;
    if (n % 8) return AGO_ERR_UNSUPPORTED;
    return from_hip(add_act(a, b, y, n, act, dt == AGO_BF16, as_stream(hip_stream)));
}

ago_status ago_scale(const void* x, void* y, long n, float alpha, ago_dtype dt, void* hip_stream) {
    const void* ps[2] = {x, y};
    ago_status st = check_ptrs(ps, 2, 2);
    if (st != AGO_OK) return st;
    if (!valid_dtype(dt)) return AGO_ERR_DTYPE;
    if (n <= 0) return AGO_ERR_SHAPE;
    if (n % 8) return AGO_ERR_UNSUPPORTED;
    return from_hip(scale(x, y, n, alpha, dt == AGO_BF16, as_stream(hip_stream)));
}

ago_status ago_softmax_rows(const void* x, void* y, long rows, int cols, ago_dtype in_dt,
                            ago_dtype out_dt, void* hip_stream) {
    const void* ps[2] = {x, y};
    ago_status st = check_ptrs(ps, 2, 2);
    if (st != AGO_OK) return st;
    if (!valid_dtype(in_dt) || !valid_dtype(out_dt)) return AGO_ERR_DTYPE;
    if (rows <= 0 || cols <= 0) return AGO_ERR_SHAPE;
    if (cols % 8 || cols > 4096 || (in_dt == AGO_BF16 && out_dt == AGO_F32)) return AGO_ERR_UNSUPPORTED;
    return from_hip(softmax_rows(x, y, rows, cols, in_dt == AGO_BF16, out_dt == AGO_BF16, as_stream(hip_stream)));
}

ago_status ago_bmm_nt(const void* a, const void* b, void* c, long batch, int M, int N, int K, float alpha,
                      ago_dtype dt, ago_dtype out_dt, void* hip_stream) {
    const void* ps[3] = {a, b, c};
    ago_status st = check_ptrs(ps, 3, 3);
    if (st != AGO_OK) return st;
    if (!valid_dtype(dt) || !valid_dtype(out_dt)) return AGO_ERR_DTYPE;
    if (batch <= 0 || M <= 0 || N <= 0 || K <= 0) return AGO_ERR_SHAPE;
    if (dt != AGO_BF16 || K % 8 || N % 8 || batch > 65535) return AGO_ERR_UNSUPPORTED;
    if (!fits31(M, N, 1, 1) || !fits31(M, K, 1, 1) || !fits31(N, K, 1, 1)) return AGO_ERR_UNSUPPORTED;
    return from_hip(bmm_nt_bf16(a, b, c, batch, M, N, K, alpha, out_dt == AGO_F32, as_stream(hip_stream)));
}

ago_status ago_bmm_nn(const void* a, const void* b, void* c, long batch, int M, int N, int K,
                      ago_dtype dt, void* hip_stream) {
    const void* ps[3] = {a, b, c};
    ago_status st = check_ptrs(ps, 3, 3);
    if (st != AGO_OK) return st;
    if (!valid_dtype(dt)) return AGO_ERR_DTYPE;
    if (batch <= 0 || M <= 0 || N <= 0 || K <= 0) return AGO_ERR_SHAPE;
    if (dt != AGO_BF16 || K % 8 || N % 8 || batch > 65535) return AGO_ERR_UNSUPPORTED;
    if (!fits31(M, N, 1, 1) || !fits31(M, K, 1, 1) || !fits31(N, K, 1, 1)) return AGO_ERR_UNSUPPORTED;
    return from_hip(bmm_nn_bf16(a, b, c, batch, M, N, K, as_stream(hip_stream)));
}

// ---------------------------------------------------------------- un-fused subgraphs
#define AGO_TRY(expr) do { ago_status _s = (expr); if (_s != AGO_OK) return _s; } while (0)

ago_status ago_unfused_invres(const void* x, const void* w1, const float* b1, const void* wd,
                              const float* bd, const void* w2, const float* b2, void* y, int N, int H,
                              int W, int Cin, int Cexp, int Cout, int stride, int residual,
                              ago_dtype dt, int epilogue_fused, void* workspace, size_t workspace_bytes,
                              void* s) {
    AGO_TRY(check_invres(x, w1, wd, w2, y, b1, bd, b2, N, H, W, Cin, Cexp, Cout, stride, residual, dt));
    const int dims[7] = {N, H, W, Cin, Cexp, Cout, stride};
    AGO_TRY(check_workspace(workspace, workspace_bytes, ago::workspace_bytes(AGO_OP_UNFUSED_INVRES, dims, 7, dt)));
    const int OH = (H - 1) / stride + 1, OW = (W - 1) / stride + 1;
    const long PE = (long)N * H * W, PO = (long)N * OH * OW;
    char* e = static_cast<char*>(workspace);
    char* d = e + (size_t)PE * Cexp * esize(dt);
    if (epilogue_fused) {
        AGO_TRY(ago_conv1x1(x, w1, b1, nullptr, e, N, H, W, Cin, Cexp, AGO_ACT_RELU6, dt, s));
        AGO_TRY(ago_dwconv3x3(e, wd, bd, d, N, H, W, Cexp, stride, AGO_ACT_RELU6, dt, s));
        AGO_TRY(ago_conv1x1(d, w2, b2, residual ? x : nullptr, y, N, OH, OW, Cexp, Cout, AGO_ACT_NONE, dt, s));
    } else {
        AGO_TRY(ago_conv1x1(x, w1, nullptr, nullptr, e, N, H, W, Cin, Cexp, AGO_ACT_NONE, dt, s));
        if (b1) AGO_TRY(ago_bias_act(e, b1, e, PE, Cexp, AGO_ACT_NONE, dt, s));
        AGO_TRY(ago_bias_act(e, nullptr, e, PE, Cexp, AGO_ACT_RELU6, dt, s));
        AGO_TRY(ago_dwconv3x3(e, wd, nullptr, d, N, H, W, Cexp, stride, AGO_ACT_NONE, dt, s));
        if (bd) AGO_TRY(ago_bias_act(d, bd, d, PO, Cexp, AGO_ACT_NONE, dt, s));
        AGO_TRY(ago_bias_act(d, nullptr, d, PO, Cexp, AGO_ACT_RELU6, dt, s));
        AGO_TRY(ago_conv1x1(d, w2, nullptr, nullptr, y, N, OH, OW, Cexp, Cout, AGO_ACT_NONE, dt, s));
        if (b2) AGO_TRY(ago_bias_act(y, b2, y, PO, Cout, AGO_ACT_NONE, dt, s));
        if (residual) AGO_TRY(ago_add_act(y, x, y, PO * Cout, AGO_ACT_NONE, dt, s));
    }
    return AGO_OK;
}

ago_status ago_unfused_conv_chain(const void* x, const void* wa, const float* ba, const void* wb,
                                  const float* bb, void* y, int N, int H, int W, int C, int residual,
                                  ago_dtype dt, int epilogue_fused, void* workspace,
                                  size_t workspace_bytes, void* s) {
    AGO_TRY(check_conv_chain(x, wa, wb, y, ba, bb, N, H, W, C, dt));
    const int dims[4] = {N, H, W, C};
    AGO_TRY(check_workspace(workspace, workspace_bytes, ago::workspace_bytes(AGO_OP_UNFUSED_CONV_CHAIN, dims, 4, dt)));
    const long P = (long)N * H * W;
    void* t = workspace;
    if (epilogue_fused) {
        AGO_TRY(ago_conv3x3(x, wa, ba, nullptr, t, N, H, W, C, C, AGO_ACT_RELU, dt, s));
        AGO_TRY(ago_conv3x3(t, wb, bb, residual ? x : nullptr, y, N, H, W, C, C, AGO_ACT_RELU, dt, s));
    } else {
        AGO_TRY(ago_conv3x3(x, wa, nullptr, nullptr, t, N, H, W, C, C, AGO_ACT_NONE, dt, s));
        if (ba) AGO_TRY(ago_bias_act(t, ba, t, P, C, AGO_ACT_NONE, dt, s));
        AGO_TRY(ago_bias_act(t, nullptr, t, P, C, AGO_ACT_RELU, dt, s));
        AGO_TRY(ago_conv3x3(t, wb, nullptr, nullptr, y, N, H, W, C, C, AGO_ACT_NONE, dt, s));
        if (bb) AGO_TRY(ago_bias_act(y, bb, y, P, C, AGO_ACT_NONE, dt, s));
        if (residual) AGO_TRY(ago_add_act(y, x, y, P * C, AGO_ACT_NONE, dt, s));
        AGO_TRY(ago_bias_act(y, nullptr, y, P, C, AGO_ACT_RELU, dt, s));
    }
    return AGO_OK;
}

ago_status ago_unfused_ffn(const void* x, const void* w1, const float* b1, const void* w2,
                           const float* b2, void* y, int M, int K, int F, int K2, ago_act act,
                           ago_dtype dt, int epilogue_fused, void* workspace, size_t workspace_bytes,
                           void* s) {
    AGO_TRY(check_ffn(x, w1, w2, y, b1, b2, M, K, F, K2, act, dt));
    const int dims[4] = {M, K, F, K2};
    AGO_TRY(check_workspace(workspace, workspace_bytes, ago::workspace_bytes(AGO_OP_UNFUSED_FFN, dims, 4, dt)));
    void* h = workspace;
    if (epilogue_fused) {
        AGO_TRY(ago_gemm(x, w1, b1, nullptr, h, M, K, F, act, dt, s));
        AGO_TRY(ago_gemm(h, w2, b2, nullptr, y, M, F, K2, AGO_ACT_NONE, dt, s));
    } else {
        AGO_TRY(ago_gemm(x, w1, nullptr, nullptr, h, M, K, F, AGO_ACT_NONE, dt, s));
        if (b1) AGO_TRY(ago_bias_act(h, b1, h, M, F, AGO_ACT_NONE, dt, s));
        if (act != AGO_ACT_NONE) AGO_TRY(ago_bias_act(h, nullptr, h, M, F, act, dt, s));
        AGO_TRY(ago_gemm(h, w2, nullptr, nullptr, y, M, F, K2, AGO_ACT_NONE, dt, s));
        if (b2) AGO_TRY(ago_bias_act(y, b2, y, M, K2, AGO_ACT_NONE, dt, s));
    }
    return AGO_OK;
}

ago_status ago_fused_attn_strided(const void* q, const void* k, const void* v, void* o, int B, int Hh,
                                  int S, int D, long long stride_b, long long stride_h, long long stride_s,
                                  float scale, ago_dtype dt, void* workspace, size_t workspace_bytes,
                                  void* hip_stream) {
    (void)workspace; (void)workspace_bytes;
    ago_status st = check_attn(q, k, v, o, B, Hh, S, D, scale, dt);
    if (st != AGO_OK) return st;
    // rows of D contiguous elements, every row start 16-byte aligned, and no two rows overlapping
    if (stride_b <= 0 || stride_h <= 0 || stride_s < D) return AGO_ERR_SHAPE;
    if (stride_b % 8 || stride_h % 8 || stride_s % 8) return AGO_ERR_ALIGN;
    return from_hip(fused_attn(q, k, v, o, B, Hh, S, scale, tile_config(AGO_OP_FUSED_ATTN), as_stream(hip_stream),
                               (long)stride_b, (long)stride_h, (long)stride_s, D));
}

ago_status ago_fused_attn_bias(const void* q, const void* k, const void* v, const void* bias, void* o, int B,
                               int Hh, int S, int D, long long bias_stride_b, long long bias_stride_h,
                               float scale, ago_dtype dt, void* workspace, size_t workspace_bytes,
                               void* hip_stream) {
    (void)workspace; (void)workspace_bytes;
    ago_status st = check_attn(q, k, v, o, B, Hh, S, D, scale, dt);
    if (st != AGO_OK) return st;
    if (!bias) return AGO_ERR_NULL;
    // a stride is 0 (broadcast) or at least the extent below it
    const long long plane = (long long)S * S;
    if (bias_stride_h != 0 && bias_stride_h < plane) return AGO_ERR_SHAPE;
    if (bias_stride_b != 0 && bias_stride_b < (bias_stride_h ? bias_stride_h * Hh : plane)) return AGO_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(bias) % 2) return AGO_ERR_ALIGN;
    if (!fits31(S, S, 1, 1)) return AGO_ERR_UNSUPPORTED;
    return from_hip(fused_attn_bias(q, k, v, bias, o, B, Hh, S, (long)bias_stride_b, (long)bias_stride_h, scale,
                                    tile_config(AGO_OP_FUSED_ATTN), as_stream(hip_stream), D));
}

ago_status ago_fused_qkv(const void* x, const void* wq, const void* wk, const void* wv, const float* bq,
                         const float* bk, const float* bv, void* q, void* k, void* v, int B, int S, int K,
                         int Hh, int D, int head_major, ago_dtype dt, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
    (void)workspace; (void)workspace_bytes;
    if (!x || !wq || !wk || !wv || !q || !k || !v) return AGO_ERR_NULL;
    if (dt != AGO_F32 && dt != AGO_BF16) return AGO_ERR_DTYPE;
    if (B <= 0 || S <= 0 || K <= 0 || Hh <= 0 || D <= 0) return AGO_ERR_SHAPE;
    if ((long long)B * S > 0x7fffffffLL || (long long)Hh * D > 0x7fffffffLL) return AGO_ERR_SHAPE;
    const void* ps[10] = {x, wq, wk, wv, q, k, v, bq, bk, bv};
    for (const void* p : ps)
        if (p && reinterpret_cast<uintptr_t>(p) % 16) return AGO_ERR_ALIGN;
    if (dt != AGO_BF16 || K % 8 || (Hh * D) % 8) return AGO_ERR_UNSUPPORTED;
    if (!fits31(B, S, K > Hh * D ? K : Hh * D, 1) || !fits31(K, Hh, D, 1)) return AGO_ERR_UNSUPPORTED;
    return from_hip(fused_qkv(x, wq, wk, wv, bq, bk, bv, q, k, v, B, S, K, Hh, D, head_major != 0,
                              as_stream(hip_stream)));
}

ago_status ago_unfused_attn(const void* q, const void* k, const void* v, void* o, int B, int Hh, int S,
                            int D, float scale, ago_dtype dt, int epilogue_fused, void* workspace,
                            size_t workspace_bytes, void* s) {
    AGO_TRY(check_attn(q, k, v, o, B, Hh, S, D, scale, dt));
    // Rows of the score / probability matrices are padded to a multiple of 8 elements (16-byte accesses)
    // in the workspace: the softmax treats the pad columns as -inf and writes them as 0, so the second
    // product may read whole 16-byte chunks of a row.
    const int Sp = (S + 7) & ~7;
    if (Sp > 4096 || !fits31(S, Sp, 1, 1) || (long)B * Hh > 65535) return AGO_ERR_UNSUPPORTED;
    const int dims[4] = {B, Hh, S, D};
    AGO_TRY(check_workspace(workspace, workspace_bytes, ago::workspace_bytes(AGO_OP_UNFUSED_ATTN, dims, 4, dt)));
    // scores stay fp32 (the softmax is an fp32 operator); the probabilities are rounded to bf16
    // because they feed a bf16 matrix product
    const long batch = (long)B * Hh;
    hipStream_t st = as_stream(s);
    void* sc = workspace;
    void* pr = static_cast<char*>(workspace) + (size_t)batch * S * Sp * 4;
    if (epilogue_fused) {
        AGO_TRY(from_hip(bmm_nt_bf16(q, k, sc, batch, S, S, D, scale, true, st, Sp)));
    } else {
        AGO_TRY(from_hip(bmm_nt_bf16(q, k, sc, batch, S, S, D, 1.0f, true, st, Sp)));
        AGO_TRY(from_hip(ago::scale(sc, sc, batch * S * Sp, scale, false, st)));
    }
    AGO_TRY(from_hip(softmax_rows(sc, pr, batch * S, S, false, true, st, Sp)));
    AGO_TRY(from_hip(bmm_nn_bf16(pr, v, o, batch, S, D, S, st, Sp)));
    return AGO_OK;
}

}  // extern "C"
