// Host-only logic behind the C ABI: argument validation, workspace sizes, tile-configuration
// state and the recompute model.  No HIP header is included here, so this translation unit also
// builds with a plain C++ compiler.
#pragma once
#include <stddef.h>
#include "../../include/ago.h"

namespace ago {

// Validators return AGO_OK or the first problem found, in the order: NULL pointers, dtype /
// activation codes, shapes, alignment, unsupported sizes, workspace.
ago_status check_invres(const void* x, const void* w1, const void* wd, const void* w2, const void* y,
                        const void* b1, const void* bd, const void* b2,
                        int N, int H, int W, int Cin, int Cexp, int Cout, int stride, int residual,
                        int dt);
ago_status check_pw_dw(const void* x, const void* w1, const void* wd, const void* y, const void* b1,
                       const void* bd, int N, int H, int W, int Cin, int Cexp, int stride, int dt);
ago_status check_dw_pw(const void* x, const void* wd, const void* w2, const void* y, const void* bd,
                       const void* b2, int N, int H, int W, int C, int Cout, int stride, int dt);
ago_status check_conv_chain(const void* x, const void* wa, const void* wb, const void* y,
                            const void* ba, const void* bb, int N, int H, int W, int C, int dt);
ago_status check_ffn(const void* x, const void* w1, const void* w2, const void* y, const void* b1,
                     const void* b2, int M, int K, int F, int K2, int act, int dt);
ago_status check_ffn_packed(const void* x, const void* w1p, const void* w2p, const void* y, const void* b1,
                            const void* b2, int M, int K, int F, int K2, int act, int dt);
ago_status check_pack_weight(const void* w, const void* wp, int K, int N, int dt);
ago_status check_gemm_packed(const void* a, const void* wp, const void* c, const void* bias, int M, int K, int N,
                             int act, int dt);
ago_status check_attn(const void* q, const void* k, const void* v, const void* o, int B, int Hh, int S,
                      int D, float scale, int dt);
ago_status check_workspace(const void* workspace, size_t have, size_t need);
ago_status check_ptrs(const void* const* ptrs, int n_required, int n_total);
bool valid_dtype(int dt);
bool valid_act(int act);
bool fits31(long long a, long long b, long long c, long long d);   // a*b*c*d < 2^31 (each factor too)

size_t workspace_bytes(int op, const int* dims, int ndims, int dt);

// Analytic planners (ago_plan.cpp): the candidate with the lowest predicted time, or the one `tile_cfg` names.
struct ChainPlan {
    int cfg, tile_h, tile_w, resident;
    long workgroups, rounds;
    double executed_upstream_macs, algorithmic_upstream_macs, predicted_us;
};
struct AttnPlan {
    int cfg, queries, key_block, stages, resident, lds_bytes;
    long workgroups, rounds;
    double executed_upstream_macs, algorithmic_upstream_macs, predicted_us;
};
struct FfnPlan {
    int rows, slice, slices, resident, fuse;
    long workgroups, rounds;
    double executed_upstream_macs, algorithmic_upstream_macs, partial_bytes, predicted_us, predicted_unfused_us;
};
bool plan_conv_chain(int N, int H, int W, int C, int tile_cfg, ChainPlan* out);
bool plan_attn(int B, int Hh, int S, int D, int tile_cfg, AttnPlan* out);
bool plan_ffn(int M, int K, int F, int K2, FfnPlan* out);
int tile_config(int op);          // current selection for a fused op (-1 = built-in)

}  // namespace ago
