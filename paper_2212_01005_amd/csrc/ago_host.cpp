// Host-only logic behind the C ABI: argument validation (runs before any HIP call), workspace
// sizes, tile-configuration state, status strings and the recompute model of Sec. III-B.
#include "ago_host.hpp"
#include <stdint.h>

namespace ago {

// from the kernel translation units (host functions)
int fused_invres_num_cfgs();
int fused_conv_chain_num_cfgs();
int fused_ffn_num_cfgs();
int fused_attn_num_cfgs();
int fused_ffn_pick_cfg(int M, int K, int F, int K2, int tile_cfg);
int fused_ffn_nsplit(int cfg, int F);
bool fused_ffn_packed_ok(int M, int K, int F, int K2);
long fused_ffn_packed_rows(int M);
int fused_ffn_packed_nsplit(int F);
int gemm_packed_variant(int M, int K, int N);
size_t fused_invres_workspace(int N, int H, int W, int Cin, int Cexp, int Cout, int stride, int ksize, bool bf16,
                              int tile_cfg, int mode);

static int g_tile_cfg[4] = {-1, -1, -1, -1};

bool valid_dtype(int dt) { return dt == AGO_F32 || dt == AGO_BF16; }
bool valid_act(int act) { return act >= AGO_ACT_NONE && act <= AGO_ACT_GELU_TANH; }
static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
// The kernels index a tensor with 32-bit element offsets inside one image / batch entry and derive grid
// sizes from int products: a tensor of 2^31 elements or more is refused rather than risked.
bool fits31(long long a, long long b, long long c, long long d) {
    const long long lim = 1LL << 31;
    long long n = a;
    for (long long f : {b, c, d}) {
        if (n >= lim || f >= lim) return false;
        n *= f;
    }
    return n < lim;
}

ago_status check_ptrs(const void* const* ptrs, int n_required, int n_total) {
    for (int i = 0; i < n_required; ++i)
        if (!ptrs[i]) return AGO_ERR_NULL;
    for (int i = 0; i < n_total; ++i)
        if (ptrs[i] && !aligned16(ptrs[i])) return AGO_ERR_ALIGN;
    return AGO_OK;
}

ago_status check_workspace(const void* workspace, size_t have, size_t need) {
    if (need == 0) return AGO_OK;
    if (!workspace || have < need) return AGO_ERR_WORKSPACE;
    if (!aligned16(workspace)) return AGO_ERR_ALIGN;
    return AGO_OK;
}

ago_status check_invres(const void* x, const void* w1, const void* wd, const void* w2, const void* y,
                        const void* b1, const void* bd, const void* b2,
                        int N, int H, int W, int Cin, int Cexp, int Cout, int stride, int residual,
                        int dt) {
    if (!x || !w1 || !wd || !w2 || !y) return AGO_ERR_NULL;
    if (!valid_dtype(dt)) return AGO_ERR_DTYPE;
    if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cexp <= 0 || Cout <= 0) return AGO_ERR_SHAPE;
    if (stride != 1 && stride != 2) return AGO_ERR_SHAPE;
    if (residual && (stride != 1 || Cin != Cout)) return AGO_ERR_SHAPE;
    const void* ps[8] = {x, w1, wd, w2, y, b1, bd, b2};
    for (const void* p : ps)
        if (p && !aligned16(p)) return AGO_ERR_ALIGN;
    if (Cin % 8 || Cexp % 16 || Cout % 8) return AGO_ERR_UNSUPPORTED;
    const int cmax = Cin > Cexp ? (Cin > Cout ? Cin : Cout) : (Cexp > Cout ? Cexp : Cout);
    if (!fits31(N, H, W, cmax)) return AGO_ERR_UNSUPPORTED;
    return AGO_OK;
}

ago_status check_pw_dw(const void* x, const void* w1, const void* wd, const void* y, const void* b1,
                       const void* bd, int N, int H, int W, int Cin, int Cexp, int stride, int dt) {
    if (!x || !w1 || !wd || !y) return AGO_ERR_NULL;
    if (!valid_dtype(dt)) return AGO_ERR_DTYPE;
    if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cexp <= 0) return AGO_ERR_SHAPE;
    if (stride != 1 && stride != 2) return AGO_ERR_SHAPE;
    const void* ps[6] = {x, w1, wd, y, b1, bd};
    for (const void* p : ps)
        if (p && !aligned16(p)) return AGO_ERR_ALIGN;
    if (Cin % 8 || Cexp % 16) return AGO_ERR_UNSUPPORTED;
    if (!fits31(N, H, W, Cin > Cexp ? Cin : Cexp)) return AGO_ERR_UNSUPPORTED;
    return AGO_OK;
}

ago_status check_dw_pw(const void* x, const void* wd, const void* w2, const void* y, const void* bd,
                       const void* b2, int N, int H, int W, int C, int Cout, int stride, int dt) {
    if (!x || !wd || !w2 || !y) return AGO_ERR_NULL;
    if (!valid_dtype(dt)) return AGO_ERR_DTYPE;
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || Cout <= 0) return AGO_ERR_SHAPE;
    if (stride != 1 && stride != 2) return AGO_ERR_SHAPE;
    const void* ps[6] = {x, wd, w2, y, bd, b2};
    for (const void* p : ps)
        if (p && !aligned16(p)) return AGO_ERR_ALIGN;
    if (C % 16 || Cout % 8) return AGO_ERR_UNSUPPORTED;
    if (!fits31(N, H, W, C > Cout ? C : Cout)) return AGO_ERR_UNSUPPORTED;
    return AGO_OK;
}

ago_status check_conv_chain(const void* x, const void* wa, const void* wb, const void* y,
                            const void* ba, const void* bb, int N, int H, int W, int C, int dt) {
    if (!x || !wa || !wb || !y) return AGO_ERR_NULL;
    if (!valid_dtype(dt)) return AGO_ERR_DTYPE;
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0) return AGO_ERR_SHAPE;
    const void* ps[6] = {x, wa, wb, y, ba, bb};
    for (const void* p : ps)
        if (p && !aligned16(p)) return AGO_ERR_ALIGN;
    if (dt != AGO_BF16 || C != 64) return AGO_ERR_UNSUPPORTED;
    if (!fits31(N, H, W, C)) return AGO_ERR_UNSUPPORTED;
    return AGO_OK;
}

ago_status check_ffn(const void* x, const void* w1, const void* w2, const void* y, const void* b1,
                     const void* b2, int M, int K, int F, int K2, int act, int dt) {
    if (!x || !w1 || !w2 || !y) return AGO_ERR_NULL;
    if (!valid_dtype(dt) || !valid_act(act)) return AGO_ERR_DTYPE;
    if (M <= 0 || K <= 0 || F <= 0 || K2 <= 0) return AGO_ERR_SHAPE;
    const void* ps[6] = {x, w1, w2, y, b1, b2};
    for (const void* p : ps)
        if (p && !aligned16(p)) return AGO_ERR_ALIGN;
    if (dt != AGO_BF16 || K % 64 || F % 8 || K2 % 8) return AGO_ERR_UNSUPPORTED;
    if (!fits31(M, K > F ? (K > K2 ? K : K2) : (F > K2 ? F : K2), 1, 1) || !fits31(K > K2 ? K : K2, F, 1, 1))
        return AGO_ERR_UNSUPPORTED;
    return AGO_OK;
}

ago_status check_ffn_packed(const void* x, const void* w1p, const void* w2p, const void* y, const void* b1,
                            const void* b2, int M, int K, int F, int K2, int act, int dt) {
    if (!x || !w1p || !w2p || !y) return AGO_ERR_NULL;
    if (!valid_dtype(dt) || !valid_act(act)) return AGO_ERR_DTYPE;
    if (M <= 0 || K <= 0 || F <= 0 || K2 <= 0) return AGO_ERR_SHAPE;
    const void* ps[6] = {x, w1p, w2p, y, b1, b2};
    for (const void* p : ps)
        if (p && !aligned16(p)) return AGO_ERR_ALIGN;
    if (dt != AGO_BF16 || !fused_ffn_packed_ok(M, K, F, K2)) return AGO_ERR_UNSUPPORTED;
    if (!fits31(M, K > F ? (K > K2 ? K : K2) : (F > K2 ? F : K2), 1, 1) || !fits31(K > K2 ? K : K2, F, 1, 1))
        return AGO_ERR_UNSUPPORTED;
    return AGO_OK;
}

ago_status check_gemm_packed(const void* a, const void* wp, const void* c, const void* bias, int M, int K, int N,
                             int act, int dt) {
    if (!a || !wp || !c) return AGO_ERR_NULL;
    if (!valid_dtype(dt) || !valid_act(act)) return AGO_ERR_DTYPE;
    if (M <= 0 || K <= 0 || N <= 0) return AGO_ERR_SHAPE;
    const void* ps[4] = {a, wp, c, bias};
    for (const void* p : ps)
        if (p && !aligned16(p)) return AGO_ERR_ALIGN;
    if (dt != AGO_BF16 || gemm_packed_variant(M, K, N) == 0) return AGO_ERR_UNSUPPORTED;
    if (!fits31(M, K > N ? K : N, 1, 1) || !fits31(K, N, 1, 1)) return AGO_ERR_UNSUPPORTED;
    return AGO_OK;
}

ago_status check_pack_weight(const void* w, const void* wp, int K, int N, int dt) {
    if (!w || !wp) return AGO_ERR_NULL;
    if (!valid_dtype(dt)) return AGO_ERR_DTYPE;
    if (K <= 0 || N <= 0) return AGO_ERR_SHAPE;
    if (!aligned16(w) || !aligned16(wp)) return AGO_ERR_ALIGN;
    if (dt != AGO_BF16 || K % 32 || N % 16 || !fits31(K, N, 1, 1)) return AGO_ERR_UNSUPPORTED;
    return AGO_OK;
}

ago_status check_attn(const void* q, const void* k, const void* v, const void* o, int B, int Hh, int S,
                      int D, float scale, int dt) {
    if (!q || !k || !v || !o) return AGO_ERR_NULL;
    if (!valid_dtype(dt)) return AGO_ERR_DTYPE;
    if (B <= 0 || Hh <= 0 || S <= 0 || D <= 0) return AGO_ERR_SHAPE;
    const void* ps[4] = {q, k, v, o};
    for (const void* p : ps)
        if (!aligned16(p)) return AGO_ERR_ALIGN;
    if (dt != AGO_BF16 || (D != 64 && D != 128) || !(scale > 0.0f)) return AGO_ERR_UNSUPPORTED;
    if (!fits31(B, Hh, S, D)) return AGO_ERR_UNSUPPORTED;
    return AGO_OK;
}

int tile_config(int op) { return (op >= 0 && op < 4) ? g_tile_cfg[op] : -1; }

size_t workspace_bytes(int op, const int* d, int nd, int dt) {
    if (!d || !valid_dtype(dt)) return 0;
    for (int i = 0; i < nd; ++i)
        if (d[i] <= 0) return 0;
    const size_t es = dt == AGO_BF16 ? 2 : 4;
    switch (op) {
        case AGO_OP_FUSED_INVRES: {       // dims N, H, W, Cin, Cexp, Cout, stride [, depthwise size]: channel-split partials
            if (nd < 7 || d[3] % 8 || d[4] % 16 || d[5] % 8) return 0;
            return fused_invres_workspace(d[0], d[1], d[2], d[3], d[4], d[5], d[6], nd > 7 ? d[7] : 3, dt == AGO_BF16,
                                          g_tile_cfg[AGO_OP_FUSED_INVRES], 0);
        }
        case AGO_OP_FUSED_DW_PW: {        // dims N, H, W, C, Cout, stride [, depthwise size]
            if (nd < 6 || d[3] % 16 || d[4] % 8) return 0;
            return fused_invres_workspace(d[0], d[1], d[2], 8, d[3], d[4], d[5], nd > 6 ? d[6] : 3, dt == AGO_BF16,
                                          g_tile_cfg[AGO_OP_FUSED_INVRES], 2);
        }
        case AGO_OP_FUSED_PW_PW: {        // dims N, H, W, Cin, Cmid, Cout: the FFN kernel on M = N H W rows
            if (nd < 6) return 0;
            const long long m = (long long)d[0] * d[1] * d[2];
            if (m >= (1LL << 31)) return 0;
            const int cfg = fused_ffn_pick_cfg((int)m, d[3], d[4], d[5], g_tile_cfg[AGO_OP_FUSED_FFN]);
            const int ns = fused_ffn_nsplit(cfg, d[4]);
            return ns > 1 ? (size_t)ns * (size_t)m * d[5] * 4 : 0;
        }
        case AGO_OP_FUSED_FFN: {
            if (nd < 4) return 0;
            const int cfg = fused_ffn_pick_cfg(d[0], d[1], d[2], d[3], g_tile_cfg[AGO_OP_FUSED_FFN]);
            const int ns = fused_ffn_nsplit(cfg, d[2]);
            return ns > 1 ? (size_t)ns * d[0] * d[3] * 4 : 0;
        }
        case AGO_OP_FUSED_FFN_PACKED: {   // fp32 partial sums [slices][rows padded to 64][K2]
            if (nd < 4 || !fused_ffn_packed_ok(d[0], d[1], d[2], d[3])) return 0;
            return (size_t)fused_ffn_packed_nsplit(d[2]) * (size_t)fused_ffn_packed_rows(d[0]) * d[3] * 4;
        }
        case AGO_OP_UNFUSED_INVRES: {     // E [N,H,W,Cexp] and D [N,OH,OW,Cexp]
            if (nd < 7) return 0;
            const size_t oh = (d[1] - 1) / d[6] + 1, ow = (d[2] - 1) / d[6] + 1;
            return ((size_t)d[0] * d[1] * d[2] + (size_t)d[0] * oh * ow) * d[4] * es;
        }
        case AGO_OP_UNFUSED_CONV_CHAIN:   // T [N,H,W,C]
            return nd < 4 ? 0 : (size_t)d[0] * d[1] * d[2] * d[3] * es;
        case AGO_OP_UNFUSED_FFN:          // hidden [M,F]
            return nd < 4 ? 0 : (size_t)d[0] * d[2] * es;
        case AGO_OP_UNFUSED_ATTN:         // scores [B,Hh,S,Sp] fp32 + probabilities in the storage type, Sp = S rounded up to 8
            return nd < 4 ? 0 : (size_t)d[0] * d[1] * d[2] * ((d[2] + 7) & ~7) * (4 + es);
        default:
            return 0;
    }
}

}  // namespace ago

extern "C" {

size_t ago_workspace_bytes(ago_op op, const int* dims, int ndims, ago_dtype dt) {
    return ago::workspace_bytes((int)op, dims, ndims, (int)dt);
}

const char* ago_status_string(ago_status s) {
    switch (s) {
        case AGO_OK: return "AGO_OK";
        case AGO_ERR_NULL: return "AGO_ERR_NULL: a required pointer is NULL";
        case AGO_ERR_SHAPE: return "AGO_ERR_SHAPE: non-positive or inconsistent dimension";
        case AGO_ERR_DTYPE: return "AGO_ERR_DTYPE: unknown dtype or activation";
        case AGO_ERR_ALIGN: return "AGO_ERR_ALIGN: pointer not 16-byte aligned";
        case AGO_ERR_UNSUPPORTED: return "AGO_ERR_UNSUPPORTED: shape or dtype not covered by the kernels";
        case AGO_ERR_WORKSPACE: return "AGO_ERR_WORKSPACE: workspace missing or too small";
        case AGO_ERR_LAUNCH: return "AGO_ERR_LAUNCH: HIP reported an error at launch";
        default: return "unknown ago_status";
    }
}

int ago_num_tile_configs(ago_op op) {
    switch (op) {
        case AGO_OP_FUSED_INVRES: return ago::fused_invres_num_cfgs();
        case AGO_OP_FUSED_CONV_CHAIN: return ago::fused_conv_chain_num_cfgs();
        case AGO_OP_FUSED_FFN: return ago::fused_ffn_num_cfgs();
        case AGO_OP_FUSED_ATTN: return ago::fused_attn_num_cfgs();
        default: return 0;
    }
}

int ago_set_tile_config(ago_op op, int config_id) {
    const int n = ago_num_tile_configs(op);
    if (n == 0 || config_id < -1 || config_id >= n) return -1;
    ago::g_tile_cfg[(int)op] = config_id;
    return 0;
}

long long ago_fused_upstream_iterations(int N, int O1, int O2, int H2, int W2, int R2, int C2,
                                        int to2, int th2, int tw2, long long* unfused) {
    if (N <= 0 || O1 <= 0 || O2 <= 0 || H2 <= 0 || W2 <= 0 || R2 <= 0 || C2 <= 0) return -1;
    if (to2 <= 0 || th2 <= 0 || tw2 <= 0 || O2 % to2 || H2 % th2 || W2 % tw2) return -1;
    if (unfused) *unfused = (long long)N * O1 * (H2 + R2 - 1) * (W2 + C2 - 1);
    // Outer loops of the downstream operator (one iteration per downstream tile) ...
    const long long outer = (long long)N * (O2 / to2) * (H2 / th2) * (W2 / tw2);
    // ... each of which recomputes the upstream tile it needs: all O1 channels of a
    // (th2 + R2 - 1) x (tw2 + C2 - 1) window.
    return outer * O1 * (th2 + R2 - 1) * (tw2 + C2 - 1);
}

}  // extern "C"
