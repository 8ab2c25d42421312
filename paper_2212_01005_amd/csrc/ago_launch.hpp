// Host-side launchers implemented next to their kernels; the C ABI in ago_api.hip validates
// arguments and then calls these.  Every launcher enqueues on `s` and returns hipGetLastError().
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <mutex>

namespace ago {

// Raises the dynamic-LDS limit of kernel Kern once per process; several host threads may make the first call
// together.  (The first call of an entry point must therefore come outside a stream capture.)
template <auto Kern>
inline hipError_t allow_dynamic_lds(int bytes) {
    static std::once_flag once;
    static hipError_t err = hipSuccess;
    std::call_once(once, [&] {
        err = hipFuncSetAttribute(reinterpret_cast<const void*>(Kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    });
    return err;
}

// un-fused operators
hipError_t gemm_bf16(const void* a, const void* b, const float* bias, const void* res, void* c, int M,
                     int K, int N, int act, hipStream_t s);
hipError_t gemm_f32(const void* a, const void* b, const float* bias, const void* res, void* c, int M,
                    int K, int N, int act, hipStream_t s);
hipError_t bmm_nt_bf16(const void* a, const void* b, void* c, long batch, int M, int N, int K,
                       float alpha, bool out_f32, hipStream_t s, int ldc = 0);   // ldc: elements per row of c (0 = N)
hipError_t bmm_nn_bf16(const void* a, const void* b, void* c, long batch, int M, int N, int K,
                       hipStream_t s, int lda = 0);   // lda: elements per row of a (0 = K), a multiple of 8; the row tail holds zeros
hipError_t dwconv3x3(const void* x, const void* w, const float* bias, void* y, int N, int H, int W,
                     int C, int stride, int act, bool bf16, hipStream_t s);
hipError_t conv3x3_bf16(const void* x, const void* w, const float* bias, const void* res, void* y,
                        int N, int H, int W, int act, hipStream_t s);
hipError_t conv3x3_bf16_tiled(const void* x, const void* w, const float* bias, const void* res, void* y,
                              int N, int H, int W, int act, hipStream_t s);   // on the fused chain's tile loop
hipError_t bias_act(const void* x, const float* bias, void* y, long P, int C, int act, bool bf16,
                    hipStream_t s);
hipError_t add_act(const void* a, const void* b, void* y, long n, int act, bool bf16, hipStream_t s);
hipError_t scale(const void* x, void* y, long n, float alpha, bool bf16, hipStream_t s);
hipError_t softmax_rows(const void* x, void* y, long rows, int cols, bool in_bf16, bool out_bf16,
                        hipStream_t s, int ld = 0);   // ld: elements per row of x and y (0 = cols), a multiple of 8; y's row tail is written as 0

// fused subgraphs
hipError_t fused_invres(const void* x, const void* w1, const float* b1, const void* wd, const float* bd,
                        const void* w2, const float* b2, void* y, int N, int H, int W, int Cin,
                        int Cexp, int Cout, int stride, int residual, bool bf16, int tile_cfg,
                        hipStream_t s, int mode = 0,    // mode 1: pw -> dw (y = D), mode 2: dw -> pw (x = E)
                        int ksize = 3,                  // depthwise kernel size, 3 or 5
                        void* workspace = nullptr, size_t ws_bytes = 0);   // enables the channel split
hipError_t fused_qkv(const void* x, const void* wq, const void* wk, const void* wv, const float* bq,
                     const float* bk, const float* bv, void* q, void* k, void* v, int B, int S, int K, int Hh,
                     int D, int head_major, hipStream_t s);
int fused_invres_plan(int N, int H, int W, int Cin, int Cexp, int Cout, int stride, int ksize, bool bf16,
                      int tile_cfg, int mode, size_t ws_bytes, int out[7], float* predicted_us);
size_t fused_invres_workspace(int N, int H, int W, int Cin, int Cexp, int Cout, int stride, int ksize, bool bf16,
                              int tile_cfg, int mode);
hipError_t fused_conv_chain(const void* x, const void* wa, const float* ba, const void* wb,
                            const float* bb, void* y, int N, int H, int W, int residual, int tile_cfg,
                            hipStream_t s);
hipError_t fused_ffn(const void* x, const void* w1, const float* b1, const void* w2, const float* b2,
                     void* y, int M, int K, int F, int K2, int act, int tile_cfg, void* workspace,
                     hipStream_t s);
hipError_t fused_attn(const void* q, const void* k, const void* v, void* o, int B, int Hh, int S,
                      float scale, int tile_cfg, hipStream_t s,
                      long stride_b = 0, long stride_h = 0, long stride_s = 0, int D = 64);   // D: 64 or 128
hipError_t fused_attn_bias(const void* q, const void* k, const void* v, const void* bias, void* o, int B, int Hh,
                           int S, long bias_sb, long bias_sh, float scale, int tile_cfg, hipStream_t s, int D = 64);   // element strides; 0 = [B][Hh][S][D]

// Instrumentation hook (see ago_profile_enable): record an event pair around the dominant kernel
// of a fused entry point.  No-ops unless profiling is enabled.
void prof_start(int op, hipStream_t s);
void prof_mid(int op, hipStream_t s);      // between the two kernels of an entry point that launches two
void prof_stop(int op, hipStream_t s);
void prof_shape(int op, unsigned grid, unsigned block);   // remembers the launch shape of the dominant kernel

// tile-configuration tables (host only)
hipError_t fused_dw_dw(const void* x, const void* wa, const float* ba, const void* wb, const float* bb,
                       void* y, int N, int H, int W, int C, int stride, bool bf16, hipStream_t s);
int fused_invres_num_cfgs();
int fused_conv_chain_num_cfgs();
// streaming (wave-specialised) FFN variant and the partial-product reduction shared by both variants
bool fused_ffn_stream_ok(int M, int K, int F, int K2);
hipError_t fused_ffn_stream(const void* x, const void* w1, const float* b1, const void* w2, const float* b2,
                            void* y, int M, int K, int F, int K2, int act, void* workspace, hipStream_t s,
                            int variant = 0);
hipError_t ffn_reduce(const float* part, const float* b2, void* y, long MK2, int K2, int nsplit, hipStream_t s,
                      long slice_stride = 0);
// matmul -> activation -> matmul on weights packed into matrix-instruction fragments (pack_weight)
bool fused_ffn_packed_ok(int M, int K, int F, int K2);
long fused_ffn_packed_rows(int M);
int fused_ffn_packed_nsplit(int F);
hipError_t pack_weight(const void* w, void* wp, int K, int N, hipStream_t s);
int gemm_packed_variant(int M, int K, int N);     // 0: the shape fits no tiling of the packed product
hipError_t gemm_packed(const void* a, const void* wp, const float* bias, void* c, int M, int K, int N, int act,
                       hipStream_t s);
hipError_t fused_ffn_packed(const void* x, const void* w1p, const float* b1, const void* w2p, const float* b2,
                            void* y, int M, int K, int F, int K2, int act, void* workspace, hipStream_t s);
int fused_ffn_num_cfgs();
int fused_attn_num_cfgs();
int fused_ffn_pick_cfg(int M, int K, int F, int K2, int tile_cfg);   // -1 = no configuration fits
int fused_ffn_nsplit(int cfg, int F);

}  // namespace ago
