/*
 * ago.h - C ABI of the MI355X (gfx950) fused-subgraph library.
 *
 * The library runs a *subgraph holding several complex operators* (convolutions,
 * matrix products; AGO, arXiv 2212.01005, Sec. II problem statement and Sec. III-B
 * "intensive operator fusion") as one fused GPU kernel that keeps the tensors on
 * the edges between the complex operators on-chip, and also exposes the same
 * subgraphs operator by operator (Sec. III-A, Figs. 3 and 4) as the un-fused
 * baselines.
 *
 * Conventions for every entry point
 *   pointers   DEVICE pointers unless the comment says "host".  The caller owns
 *              every buffer; the library never allocates or frees device memory.
 *              All tensor pointers must be 16-byte aligned.  Outputs must not
 *              alias inputs unless stated.
 *   layouts    activations NHWC ([N][H][W][C], C fastest); 1x1 weights [Cin][Cout];
 *              depthwise weights [3][3][C]; dense 3x3 weights [3][3][Cin][Cout];
 *              GEMM operands row-major; attention tensors [B][Hh][S][D].
 *   dtypes     `dt` is the storage type of activations and weights (AGO_F32 or
 *              AGO_BF16).  Biases are always fp32 and may be NULL (= no bias).
 *              bf16 paths accumulate, add biases, apply activations, residuals
 *              and softmax in fp32; on-chip intermediates that feed a bf16 matrix
 *              instruction are rounded to bf16 (nearest even).
 *   padding    spatial convolutions use zero padding 1; for the second operator
 *              of a chain the *intermediate* tensor is what is padded with zeros.
 *   execution  asynchronous on `hip_stream` (a hipStream_t passed as void*;
 *              NULL = the default stream); the call returns after enqueue.
 *   errors     return codes only.  Argument validation happens on the host
 *              before any HIP call; AGO_ERR_LAUNCH reports a failed launch.
 *              A shape the kernels cannot run returns AGO_ERR_UNSUPPORTED,
 *              never a wrong answer.  That includes any tensor (an on-chip
 *              intermediate counted at full size) of 2^31 elements or more:
 *              offsets inside a tensor are 32-bit.
 *   workspace  scratch for cross-workgroup partial results; size from
 *              ago_workspace_bytes().  May be NULL when that size is 0.
 */
#ifndef AGO_H
#define AGO_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    AGO_OK = 0,
    AGO_ERR_NULL = 1,         /* a required pointer is NULL */
    AGO_ERR_SHAPE = 2,        /* non-positive or inconsistent dimension */
    AGO_ERR_DTYPE = 3,        /* unknown dtype / activation code */
    AGO_ERR_ALIGN = 4,        /* pointer not 16-byte aligned */
    AGO_ERR_UNSUPPORTED = 5,  /* valid request the kernels do not cover */
    AGO_ERR_WORKSPACE = 6,    /* workspace missing or too small */
    AGO_ERR_LAUNCH = 7        /* HIP reported an error at launch */
} ago_status;

typedef enum { AGO_F32 = 0, AGO_BF16 = 1 } ago_dtype;
typedef enum { AGO_ACT_NONE = 0, AGO_ACT_RELU = 1, AGO_ACT_RELU6 = 2, AGO_ACT_GELU_TANH = 3 } ago_act;
typedef enum {
    AGO_OP_FUSED_INVRES = 0, AGO_OP_FUSED_CONV_CHAIN = 1, AGO_OP_FUSED_FFN = 2, AGO_OP_FUSED_ATTN = 3,
    AGO_OP_UNFUSED_INVRES = 4, AGO_OP_UNFUSED_CONV_CHAIN = 5, AGO_OP_UNFUSED_FFN = 6, AGO_OP_UNFUSED_ATTN = 7,
    AGO_OP_FUSED_PW_DW = 8, AGO_OP_FUSED_DW_PW = 9, AGO_OP_FUSED_PW_PW = 10, AGO_OP_FUSED_DW_DW = 11,
    AGO_OP_FUSED_FFN_PACKED = 12
} ago_op;

/* ------------------------------------------------------------------------- */
/* Fused subgraphs (Sec. III-B): several complex operators, one kernel.        */
/* ------------------------------------------------------------------------- */

/* pointwise -> depthwise -> pointwise (the pw->dw and dw->pw pairs of Sec. III-B,
 * Fig. 7a/7b; MobileNetV2 / MNasNet blocks of Sec. VI):
 *   E = relu6(x * w1 + b1)              1x1 conv, Cin -> Cexp, E := 0 outside the image
 *   D = relu6(dw3x3(E, wd, stride) + bd)
 *   y = D * w2 + b2 (+ x if residual)   1x1 conv, Cexp -> Cout
 * x:[N,H,W,Cin] w1:[Cin,Cexp] wd:[3,3,Cexp] w2:[Cexp,Cout] y:[N,OH,OW,Cout],
 * OH = (H-1)/stride + 1.  stride is 1 or 2.  residual != 0 requires stride == 1 and
 * Cin == Cout.  Requires Cin % 8 == 0, Cexp % 16 == 0, Cout % 8 == 0 (else UNSUPPORTED).
 * workspace is optional.  With ago_workspace_bytes(AGO_OP_FUSED_INVRES, {N,H,W,Cin,Cexp,Cout,stride
 * [,ksize]}) bytes of it, a wide block on few pixels (e.g. 7x7x960 at batch 1, a single tile) is cut
 * along the expanded channels as well: each workgroup takes one slice of the projection's reduction
 * (the "downstream pointwise" rule of Fig. 7b with the slices spread over the chip), writes an fp32
 * partial, and a second small kernel adds the partials, b2 and the residual.  Without (or with too
 * little) workspace one workgroup walks all slices of its tile: same result, slower on such shapes. */
ago_status ago_fused_invres(const void* x, const void* w1, const float* b1,
                            const void* wd, const float* bd,
                            const void* w2, const float* b2, void* y,
                            int N, int H, int W, int Cin, int Cexp, int Cout,
                            int stride, int residual, ago_dtype dt,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same block with a ksize x ksize depthwise, zero padding (ksize-1)/2 (the 5x5 depthwise layers
 * of the MNasNet blocks among the networks of Sec. VI): wd:[ksize,ksize,Cexp], everything else as
 * above.  ksize is 3 or 5 (else UNSUPPORTED).  The halo of E that a tile recomputes is (ksize-1)/2
 * pixels wide (the re-computation factor of Fig. 7a grows accordingly). */
ago_status ago_fused_invres_k(const void* x, const void* w1, const float* b1,
                              const void* wd, const float* bd,
                              const void* w2, const float* b2, void* y,
                              int N, int H, int W, int Cin, int Cexp, int Cout,
                              int stride, int ksize, int residual, ago_dtype dt,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): ago_fused_invres_k with the channel-split partial sums kept in a
 * buffer the library owns (a file-scope device array of AGO_NOALLOC_SCRATCH_BYTES; every GPU the library
 * runs on holds its own copy until the process ends) instead of a caller workspace.  The call allocates
 * and frees nothing.  Same arguments, result and restrictions as ago_fused_invres_k given the workspace
 * ago_workspace_bytes(AGO_OP_FUSED_INVRES, ...) asks for; shapes for which that size exceeds
 * AGO_NOALLOC_SCRATCH_BYTES return AGO_ERR_WORKSPACE before any GPU work.  All calls on one GPU share
 * the buffer (every launch overwrites what it later reads, nothing has to be cleared): two such calls
 * that overlap in time on one GPU (different streams or host threads) race; calls ordered on one stream
 * do not.  The first call on a device looks up the buffer's address (hipGetSymbolAddress). */
#define AGO_NOALLOC_SCRATCH_BYTES ((size_t)4 << 20)
ago_status ago_fused_invres_noalloc(const void* x, const void* w1, const float* b1,
                                    const void* wd, const float* bd,
                                    const void* w2, const float* b2, void* y,
                                    int N, int H, int W, int Cin, int Cexp, int Cout,
                                    int stride, int ksize, int residual, ago_dtype dt,
                                    void* hip_stream);

/* Host-only: the tiling ago_fused_invres[_k] would launch for this shape (no GPU call).  The tile
 * is the candidate with the lowest predicted time of a cost model fitted to MI355X measurements
 * (the tile-size trade-off of Sec. III-B / Fig. 7a: re-computed halo against parallelism), or the
 * one set with ago_set_tile_config (tile candidate + 16 x channel-split option).  workspace_bytes: what
 * the launch would be given (plans whose partials need more are not considered).  plan (host, 7 ints):
 * candidate index, tile rows, tile columns of output pixels, chunks of expanded channels one workgroup
 * walks, channels per chunk, LDS bytes, workgroups per tile (1 = no channel split).
 * predicted_us (host, may be NULL): the model's time in microseconds. */
ago_status ago_fused_invres_plan(int N, int H, int W, int Cin, int Cexp, int Cout, int stride, int ksize,
                                 ago_dtype dt, size_t workspace_bytes, int plan[7], float* predicted_us);

/* The two-operator pairs of the block as calls of their own (the micro-benchmark pairs of
 * Sec. VI, Fig. 13: pw->dw, dw->pw, dw->dw, pw->pw).  Same kernels, conventions and restrictions as the
 * entry points they are cut from; tile configurations follow AGO_OP_FUSED_INVRES / _FFN.
 *   ago_fused_pw_dw   y = relu6(dw3x3(relu6(x * w1 + b1), wd, stride) + bd)       (Fig. 7a)
 *                     x:[N,H,W,Cin] w1:[Cin,Cexp] wd:[3,3,Cexp] y:[N,OH,OW,Cexp]; the expanded
 *                     tensor is 0 outside the image.  Cin % 8 == 0, Cexp % 16 == 0.
 *   ago_fused_dw_pw   y = relu6(dw3x3(x, wd, stride) + bd) * w2 + b2                (Fig. 7b)
 *                     x:[N,H,W,C] wd:[3,3,C] w2:[C,Cout] y:[N,OH,OW,Cout].  C % 16 == 0, Cout % 8 == 0.
 *                     Optional workspace as for ago_fused_invres, size from
 *                     ago_workspace_bytes(AGO_OP_FUSED_DW_PW, {N,H,W,C,Cout,stride[,ksize]}).
 *   ago_fused_pw_dw_k, ago_fused_dw_pw_k   the same two pairs with a ksize x ksize depthwise (3 or 5,
 *                     zero padding (ksize-1)/2, wd:[ksize,ksize,C]): the pairs of the 5x5 blocks.
 *   ago_fused_dw_dw   y = relu6(dw3x3(relu6(dw3x3(x, wa, stride) + ba), wb, 1) + bb)  (Fig. 7a twice)
 *                     x:[N,H,W,C] wa,wb:[3,3,C] y:[N,OH,OW,C]; the intermediate is 0 outside its
 *                     image.  C % 4 == 0.  Vector ALUs only.
 *   ago_fused_pw_pw   y = act(x * w1 + b1) * w2 + b2 on NHWC tensors: ago_fused_ffn with
 *                     M = N H W, K = Cin, F = Cmid, K2 = Cout (bf16; same divisibility rules);
 *                     workspace size from ago_workspace_bytes(AGO_OP_FUSED_PW_PW,
 *                     {N,H,W,Cin,Cmid,Cout}).  The paper's caveat applies: this pair moves
 *                     more bytes fused than un-fused when N H W is small (Sec. VI-C, Fig. 13d). */
ago_status ago_fused_pw_dw(const void* x, const void* w1, const float* b1,
                           const void* wd, const float* bd, void* y,
                           int N, int H, int W, int Cin, int Cexp, int stride, ago_dtype dt,
                           void* workspace, size_t workspace_bytes, void* hip_stream);
ago_status ago_fused_pw_dw_k(const void* x, const void* w1, const float* b1,
                             const void* wd, const float* bd, void* y,
                             int N, int H, int W, int Cin, int Cexp, int stride, int ksize, ago_dtype dt,
                             void* workspace, size_t workspace_bytes, void* hip_stream);
ago_status ago_fused_dw_pw_k(const void* x, const void* wd, const float* bd,
                             const void* w2, const float* b2, void* y,
                             int N, int H, int W, int C, int Cout, int stride, int ksize, ago_dtype dt,
                             void* workspace, size_t workspace_bytes, void* hip_stream);
ago_status ago_fused_dw_pw(const void* x, const void* wd, const float* bd,
                           const void* w2, const float* b2, void* y,
                           int N, int H, int W, int C, int Cout, int stride, ago_dtype dt,
                           void* workspace, size_t workspace_bytes, void* hip_stream);
ago_status ago_fused_dw_dw(const void* x, const void* wa, const float* ba,
                           const void* wb, const float* bb, void* y,
                           int N, int H, int W, int C, int stride, ago_dtype dt,
                           void* workspace, size_t workspace_bytes, void* hip_stream);
ago_status ago_fused_pw_pw(const void* x, const void* w1, const float* b1,
                           const void* w2, const float* b2, void* y,
                           int N, int H, int W, int Cin, int Cmid, int Cout, ago_act act, ago_dtype dt,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/* conv3x3 -> conv3x3 (general convolution downstream, Sec. III-B Fig. 5 and the
 * recompute analysis that follows it), fused with halo recompute:
 *   T = relu(conv3x3(x, wa) + ba), T := 0 outside the image
 *   y = relu(conv3x3(T, wb) + bb (+ x if residual))
 * x,y:[N,H,W,C]  wa,wb:[3,3,C,C].  bf16 only; C must be 64 (else UNSUPPORTED). */
ago_status ago_fused_conv_chain(const void* x, const void* wa, const float* ba,
                                const void* wb, const float* bb, void* y,
                                int N, int H, int W, int C, int residual, ago_dtype dt,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/* matmul -> matmul (pw->pw; a matrix product is a pointwise convolution, Sec. III-B):
 *   y = act(x w1 + b1) w2 + b2
 * x:[M,K] w1:[K,F] w2:[F,K2] y:[M,K2].  bf16 only.  The hidden activation never
 * leaves the chip; partial sums over slices of F go through `workspace`.
 * Requires K % 64 == 0, F % 8 == 0, K2 % 8 == 0 (else UNSUPPORTED); F and K2 need not be multiples of
 * the kernel's 384-wide hidden slices and column blocks. */
ago_status ago_fused_ffn(const void* x, const void* w1, const float* b1,
                         const void* w2, const float* b2, void* y,
                         int M, int K, int F, int K2, ago_act act, ago_dtype dt,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same chain on weights re-laid out once, ahead of time (weights are constants of a network; the
 * paper's tuner likewise chooses data layouts, Sec. III).  ago_pack_weight is the separate call that
 * produces the layout; its cost is a one-time cost per weight tensor and bench.py reports it.
 *   ago_packed_weight_bytes(K, N)  bytes of the packed copy of a [K,N] bf16 matrix (= K N 2), 0 if the
 *                                  matrix cannot be packed (needs K % 32 == 0 and N % 16 == 0).
 *   ago_pack_weight(w, wp, K, N)   w:[K,N] row-major bf16 (device) -> wp (device, that many bytes): the
 *                                  matrix as fragments of the 16x16x32 matrix instruction, fragment
 *                                  (ks, nt) = rows 32 ks.., columns 16 nt.. stored [ks][nt][64 lanes][8],
 *                                  lane l holding w[32 ks + 8 (l / 16) + e][16 nt + l % 16], e = 0..7.
 *   ago_fused_ffn_packed           y = act(x w1 + b1) w2 + b2 with w1p = packed w1 [K,F], w2p = packed
 *                                  w2 [F,K2]; x, y, biases as for ago_fused_ffn.  Requires K % 64 == 0,
 *                                  K <= 1264, F % 64 == 0, K2 % 16 == 0 (else UNSUPPORTED).  workspace is
 *                                  required: ago_workspace_bytes(AGO_OP_FUSED_FFN_PACKED, {M,K,F,K2})
 *                                  bytes (fp32 partial sums per 384-wide hidden slice, rows padded to 64).
 * The kernel loads weight fragments from the L2 straight into registers, so the weights never pass
 * through LDS; results agree with ago_fused_ffn up to the order of the fp32 summation. */
/* The un-fused counterparts on packed weights (Fig. 3 / Fig. 4: one kernel per complex operator, its bias and
 * activation in the epilogue), so that fused and un-fused can be compared on the same weight layout:
 *   ago_gemm_packed          c = act(a wp + bias), a:[M,K] c:[M,N] bf16 row-major, wp = packed [K,N].  Tilings:
 *                            128 x 192 (needs N % 192 == 0, K % 128 == 0) or 64 x 96 with the reduction split
 *                            over the waves (N % 96 == 0, K % 512 == 0); other shapes UNSUPPORTED.
 *   ago_unfused_ffn_packed   the chain as two such products; workspace = the hidden tensor,
 *                            ago_workspace_bytes(AGO_OP_UNFUSED_FFN, {M,K,F,K2}). */
size_t ago_packed_weight_bytes(int K, int N);
/* Host-only: 1 when ago_gemm_packed has a tiling for an [M,K] x [K,N] product, else 0. */
int ago_gemm_packed_supported(int M, int K, int N);
ago_status ago_gemm_packed(const void* a, const void* wp, const float* bias, void* c,
                           int M, int K, int N, ago_act act, ago_dtype dt, void* hip_stream);
ago_status ago_unfused_ffn_packed(const void* x, const void* w1p, const float* b1,
                                  const void* w2p, const float* b2, void* y,
                                  int M, int K, int F, int K2, ago_act act, ago_dtype dt,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);
ago_status ago_pack_weight(const void* w, void* wp, int K, int N, ago_dtype dt, void* hip_stream);
ago_status ago_fused_ffn_packed(const void* x, const void* w1p, const float* b1,
                                const void* w2p, const float* b2, void* y,
                                int M, int K, int F, int K2, ago_act act, ago_dtype dt,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/* matmul -> simple operators -> matmul (the attention chain of Sec. VI-C):
 *   o = softmax_rows(scale * q k^T) v      per (batch, head), fp32 softmax
 * q,k,v,o:[B,Hh,S,D].  bf16 only; D must be 64 or 128 (else UNSUPPORTED); any S >= 1. */
ago_status ago_fused_attn(const void* q, const void* k, const void* v, void* o,
                          int B, int Hh, int S, int D, float scale, ago_dtype dt,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same attention chain on tensors whose rows are laid out by strides (in elements, the same
 * for q, k, v and o): row s of (batch b, head h) starts at b * stride_b + h * stride_h +
 * s * stride_s and holds D contiguous elements.  [B][Hh][S][D] is (Hh S D, S D, D); the
 * projection output layout [B][S][Hh][D] is (S Hh D, D, Hh D), which folds the transposes that
 * surround the chain into its addressing (Sec. VI-C counts those reshapes / transposes among the
 * simple operators between the two products).  Strides must be positive multiples of 8,
 * stride_s >= D (else SHAPE / ALIGN); rows must not overlap (not checked). */
ago_status ago_fused_attn_strided(const void* q, const void* k, const void* v, void* o,
                                  int B, int Hh, int S, int D,
                                  long long stride_b, long long stride_h, long long stride_s,
                                  float scale, ago_dtype dt,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* The attention chain with one more simple operator between the products (Sec. VI-C: the chain is
 * matmul -> simple operators -> matmul): an elementwise add of a bias or mask ahead of the softmax,
 *   o = softmax_rows(scale * q k^T + bias) v
 * q,k,v,o:[B,Hh,S,D] contiguous, bf16, D = 64 or 128.  bias (device, bf16): element (b, h, i, j) at
 * bias[b * bias_stride_b + h * bias_stride_h + i * S + j]; a stride of 0 broadcasts over that
 * dimension (a [1,Hh,S,S] relative-position table, a [B,1,S,S] padding mask), otherwise
 * bias_stride_h >= S*S and bias_stride_b >= Hh * bias_stride_h (else SHAPE).  The bias is not scaled.
 * Large negative finite values (or -inf) mask keys; a row whose keys are all -inf is undefined (NaN).
 * Rows are fetched with 16-byte loads when S and both strides are multiples of 8 and the base is
 * 16-byte aligned, element by element otherwise. */
ago_status ago_fused_attn_bias(const void* q, const void* k, const void* v, const void* bias, void* o,
                               int B, int Hh, int S, int D,
                               long long bias_stride_b, long long bias_stride_h,
                               float scale, ago_dtype dt,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* Sibling fusion (Sec. III: operators that share an input are fused into one subgraph): the three
 * projections of an attention layer in one kernel,
 *   q = x wq + bq,  k = x wk + bk,  v = x wv + bv
 * x:[B*S,K]  wq,wk,wv:[K,Hh*D]  bq,bk,bv:[Hh*D] fp32 or NULL.  Outputs (device, written in full):
 * head_major != 0: [B,Hh,S,D], the layout ago_fused_attn reads (the transpose after the projections
 * is folded into the store); head_major == 0: [B,S,Hh,D] = [B*S, Hh*D], the layout
 * ago_fused_attn_strided reads.  bf16 only; K % 8 == 0 and (Hh*D) % 8 == 0 (else UNSUPPORTED). */
ago_status ago_fused_qkv(const void* x, const void* wq, const void* wk, const void* wv,
                         const float* bq, const float* bk, const float* bv,
                         void* q, void* k, void* v,
                         int B, int S, int K, int Hh, int D, int head_major, ago_dtype dt,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------- */
/* Un-fused per-operator kernels (Sec. III-A).  With bias == NULL and           */
/* act == AGO_ACT_NONE each is exactly one operator (Fig. 3); with a bias /     */
/* activation it is the conventional epilogue fusion of Fig. 4.                 */
/* ------------------------------------------------------------------------- */

/* c = act(a b + bias + res).  a:[M,K] b:[K,N] c,res:[M,N] bias:[N]; bias and res may be NULL.
 * K % 8 == 0, N % 8 == 0. */
ago_status ago_gemm(const void* a, const void* b, const float* bias, const void* res, void* c,
                    int M, int K, int N, ago_act act, ago_dtype dt, void* hip_stream);
/* Pointwise convolution = ago_gemm with M = N*H*W (Sec. III-B). x:[N,H,W,Cin] w:[Cin,Cout]. */
ago_status ago_conv1x1(const void* x, const void* w, const float* bias, const void* res, void* y,
                       int N, int H, int W, int Cin, int Cout, ago_act act, ago_dtype dt,
                       void* hip_stream);
/* y = act(dw3x3(x, w, stride, pad 1) + bias).  C % 8 == 0. */
ago_status ago_dwconv3x3(const void* x, const void* w, const float* bias, void* y,
                         int N, int H, int W, int C, int stride, ago_act act, ago_dtype dt,
                         void* hip_stream);
/* y = act(conv3x3(x, w, pad 1) + bias + res).  res may be NULL.  bf16, Cin == Cout == 64. */
ago_status ago_conv3x3(const void* x, const void* w, const float* bias, const void* res, void* y,
                       int N, int H, int W, int Cin, int Cout, ago_act act, ago_dtype dt,
                       void* hip_stream);
/* y[p][c] = act(x[p][c] + bias[c]); bias may be NULL; y may alias x.  C % 8 == 0. */
ago_status ago_bias_act(const void* x, const float* bias, void* y, long P, int C,
                        ago_act act, ago_dtype dt, void* hip_stream);
/* y = act(a + b) elementwise; y may alias a.  n % 8 == 0. */
ago_status ago_add_act(const void* a, const void* b, void* y, long n,
                       ago_act act, ago_dtype dt, void* hip_stream);
/* y = alpha * x elementwise; y may alias x.  n % 8 == 0. */
ago_status ago_scale(const void* x, void* y, long n, float alpha, ago_dtype dt, void* hip_stream);
/* Row softmax (max-subtracted, fp32 inside).  x has type in_dt, y type out_dt; supported pairs:
 * (bf16,bf16), (f32,f32), (f32,bf16).  y may alias x when the types are equal.
 * cols % 8 == 0, cols <= 4096. */
ago_status ago_softmax_rows(const void* x, void* y, long rows, int cols, ago_dtype in_dt,
                            ago_dtype out_dt, void* hip_stream);
/* c[i] = alpha * a[i] b[i]^T.  a:[batch,M,K] b:[batch,N,K] bf16; c:[batch,M,N] of type out_dt
 * (fp32 keeps attention scores unrounded for the fp32 softmax). */
ago_status ago_bmm_nt(const void* a, const void* b, void* c, long batch, int M, int N, int K,
                      float alpha, ago_dtype dt, ago_dtype out_dt, void* hip_stream);
/* c[i] = a[i] b[i].  a:[batch,M,K] b:[batch,K,N] c:[batch,M,N].  bf16. */
ago_status ago_bmm_nn(const void* a, const void* b, void* c, long batch, int M, int N, int K,
                      ago_dtype dt, void* hip_stream);

/* The same four subgraphs run operator by operator on the kernels above, with every
 * intermediate tensor written to `workspace` (device) and read back by the next kernel.
 * epilogue_fused == 0: one kernel per operator, simple operators included (Fig. 3);
 * epilogue_fused != 0: each complex operator with its bias/activation/residual fused
 * (Fig. 4, the paper's "conventional fusion").  Arguments as in the fused calls.
 * ago_unfused_attn takes any S <= 4096: the rows of the score and probability matrices in the
 * workspace are padded to a multiple of 8 elements, the pad columns count as -inf in the softmax. */
ago_status ago_unfused_invres(const void* x, const void* w1, const float* b1,
                              const void* wd, const float* bd,
                              const void* w2, const float* b2, void* y,
                              int N, int H, int W, int Cin, int Cexp, int Cout,
                              int stride, int residual, ago_dtype dt, int epilogue_fused,
                              void* workspace, size_t workspace_bytes, void* hip_stream);
ago_status ago_unfused_conv_chain(const void* x, const void* wa, const float* ba,
                                  const void* wb, const float* bb, void* y,
                                  int N, int H, int W, int C, int residual, ago_dtype dt,
                                  int epilogue_fused,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);
ago_status ago_unfused_ffn(const void* x, const void* w1, const float* b1,
                           const void* w2, const float* b2, void* y,
                           int M, int K, int F, int K2, ago_act act, ago_dtype dt,
                           int epilogue_fused,
                           void* workspace, size_t workspace_bytes, void* hip_stream);
ago_status ago_unfused_attn(const void* q, const void* k, const void* v, void* o,
                            int B, int Hh, int S, int D, float scale, ago_dtype dt,
                            int epilogue_fused,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------- */
/* Host-side helpers (no GPU work).                                            */
/* ------------------------------------------------------------------------- */

/* Bytes of workspace the given entry point needs for the given dimensions
 * (`dims` is a host array holding the call's integer shape arguments in order,
 * e.g. {M,K,F,K2} for the FFN or {N,H,W,Cin,Cexp,Cout,stride} for the inverted
 * residual).  Returns 0 when none is needed or the arguments are invalid. */
size_t ago_workspace_bytes(ago_op op, const int* dims, int ndims, ago_dtype dt);

/* Static string naming a status code. */
const char* ago_status_string(ago_status s);

/* Select a tile configuration for a fused entry point (hook for the offline tile-size
 * sweep that stands in for the paper's schedule search).  config_id = -1 restores the
 * built-in choice.  Returns 0, or -1 for an unknown op / id. */
int ago_set_tile_config(ago_op op, int config_id);
/* Number of selectable tile configurations for `op` (0 for an unknown op). */
int ago_num_tile_configs(ago_op op);

/* Instrumentation for benchmarks.  ago_profile_enable(capacity > 0) makes every fused entry point
 * record a HIP event pair on its launch stream around its dominant kernel (the last `capacity`
 * calls per entry point are kept; capacity <= 0 switches it off and frees the events; at most
 * 4096).  ago_profile_read waits for the recorded calls of `op` (one of the four AGO_OP_FUSED_*),
 * writes their summed kernel time in milliseconds and their number to the host pointers, and
 * clears the record.  ago_profile_select restricts the recording to the entry points whose bit
 * (1u << AGO_OP_FUSED_*) is set in op_mask (default: all four); an event pair costs a few
 * microseconds on the stream, so a benchmark brackets only the kernel it reports.  All three
 * return 0, or -1 on misuse / a HIP error.  Not thread-safe. */
int ago_profile_enable(int capacity);
int ago_profile_select(unsigned op_mask);
int ago_profile_read(ago_op op, float* total_ms, int* count);
/* The same, and first_kernel_ms (host, may be NULL): the part of total_ms up to the end of the entry point's first
 * kernel, for entry points that launch two (the FFN chain with several hidden slices: streaming kernel, then the
 * partial-sum reduction); equal to total_ms otherwise. */
int ago_profile_read_split(ago_op op, float* total_ms, float* first_kernel_ms, int* count);
/* Average elapsed time in milliseconds of `pairs` (1..1024) event pairs recorded back to back on
 * `hip_stream` with nothing between them: the fixed cost an event pair adds to what it brackets.
 * Synchronises on the events.  Returns a negative value on misuse / a HIP error. */
float ago_profile_event_overhead_ms(void* hip_stream, int pairs);
/* Launch floors for the latency-bound configurations.  ago_profile_last_launch writes the grid and
 * workgroup size (in workgroups / threads) that the dominant kernel of fused entry point `op` was
 * last launched with (-1 if it has not run yet); ago_bench_empty_kernel enqueues a kernel that does
 * nothing with that shape on `hip_stream`, so a benchmark can report what launching alone costs.
 * Both return 0, or -1 on misuse / a HIP error. */
int ago_profile_last_launch(ago_op op, int* grid, int* block);
int ago_bench_empty_kernel(int grid, int block, void* hip_stream);
/* Measured matrix-core peak: enqueues a kernel of matrix instructions only (one workgroup of eight waves per compute
 * unit, six independent accumulators per wave, `iters` rounds; AGO_BF16: 32x32x16 bf16, AGO_F32: 32x32x2 fp32) and
 * writes the FLOPs it executes to *flops (host).  out: device scratch of at least compute units x 2048 bytes.
 * Time it with events: FLOPs / time is what bench.py reports as the measured peak beside the data-sheet one.
 * (The measured memory peak uses ago_scale with alpha = 1 as a plain copy.) */
int ago_bench_mfma_kernel(ago_dtype dt, int iters, void* out, size_t out_bytes, double* flops, void* hip_stream);

int ago_fused_ffn_pays(int M, int K, int F, int K2);

/* Host-only planners for the other three fused kernels (no GPU call): the tile candidate a launch would use, chosen
 * by an explicit time model whose recompute term is the redundancy algebra of Sec. III-B,
 *     upstream work = | GS2/TS2 x (GS1/TS1 - GS2/TS2) | * | TS1 |
 * (downstream tile loops x upstream loops the downstream nest lacks x upstream tile), the rest being counts of what
 * the kernels execute times rates measured on an MI355X.  ago_set_tile_config pins the candidate instead.
 * plan (host, 8 ints):
 *   conv chain  {candidate, tile rows, tile columns, workgroups, workgroups resident per compute unit, rounds, 0, 1}
 *   attention   {candidate, query rows per workgroup, keys per block, workgroups, resident, rounds, LDS bytes, 1}
 *   FFN         {candidate, rows per workgroup, hidden units per slice, workgroups, resident, rounds, slices,
 *                fuse (1) or run the two products with fused epilogues (0)}
 * recompute (host, may be NULL): executed / algorithmic multiply-adds of the upstream operator under that tiling:
 * (TH+2)(TW+2) tiles / (N H W) for the 3x3 chain (the |TS2| < |TS1| case of Sec. III-B; 1.469 for 7 x 14 tiles of a
 * 56 x 56 image), exactly 1 for the two "downstream pointwise" tilings of Fig. 7b.
 * predicted_us (host, may be NULL): the model's time for the fused launch; predicted_unfused_us: for the two
 * un-fused products.  ago_fused_ffn_pays returns the FFN plan's fuse decision (1 / 0; -1 on non-positive sizes):
 * with few rows the fused kernel wins; once the rows fill the chip several times over, the fp32 partial sums of the
 * hidden slices cost more than writing the hidden tensor once (the paper's own caveat for pw -> pw, Sec. VI-C). */
ago_status ago_fused_conv_chain_plan(int N, int H, int W, int C, int plan[8], double* recompute, float* predicted_us);
ago_status ago_fused_attn_plan(int B, int Hh, int S, int D, int plan[8], double* recompute, float* predicted_us);
ago_status ago_fused_ffn_plan(int M, int K, int F, int K2, int plan[8], double* recompute, float* predicted_us,
                              float* predicted_unfused_us);

/* Redundancy model of Sec. III-B: number of times the upstream reduction body runs
 * when a conv R1xC1 (I -> O1) is fused under a downstream conv R2xC2 (O1 -> O2) whose
 * output is tiled (to2, th2, tw2) on (O2, H2, W2), no padding, stride 1 (the setting of
 * Fig. 5).  `unfused` (host pointer, may be NULL) receives the count without fusion,
 * N*O1*(H2+R2-1)*(W2+C2-1).  Both counts exclude the I*R1*C1 factor of the reduction
 * itself.  Tile sizes must divide the dimensions; returns -1 otherwise. */
long long ago_fused_upstream_iterations(int N, int O1, int O2, int H2, int W2, int R2, int C2,
                                        int to2, int th2, int tw2, long long* unfused);

/* ------------------------------------------------------------------------- */
/* Graph frontend, host only (Sec. IV, V): which operators form one subgraph.  */
/* No GPU call; every pointer is a host pointer owned by the caller.            */
/* Nodes are 0..n_nodes-1; edge e goes from edge_src[e] to edge_dst[e] (a      */
/* tensor produced by the source operator and consumed by the destination).     */
/* Self-loops, out-of-range ids and cyclic edge sets give AGO_ERR_SHAPE.        */
/* ------------------------------------------------------------------------- */

/* Eq. 1: w = c * prod_l log(s_l) + b over the extents s_l of the operator's loop nest (natural
 * logarithm; b when there are no loops; NaN when an extent is < 1). */
double ago_graph_op_weight(const int* loop_extents, int n_loops, double c, double b);

/* Topological stage (Sec. IV-B): stage[v] = number of nodes on the longest path from a root to v
 * (roots have stage 1). */
ago_status ago_graph_topological_stage(int n_nodes, int n_edges, const int* edge_src, const int* edge_dst,
                                       int* stage);

/* Function Cluster of the graph-partition algorithm (Sec. IV-B): repeatedly take the heaviest
 * candidate (hyper) node v and merge it with the lightest node u of its affix set (a neighbour whose
 * topological stage differs by one) for which w_v + w_u < td; a candidate without such a partner
 * leaves the candidate set; edges and stages are updated after every merge.  The result is an
 * acyclic partition whose merged subgraphs weigh less than td.
 * weight:[n_nodes] >= 0.  is_complex:[n_nodes] (0/1) and max_complex > 0 additionally cap the number
 * of complex operators per subgraph (max_complex <= 0: no cap, is_complex may be NULL).
 * subgraph_of:[n_nodes] out, subgraphs numbered from 0 in order of their smallest node id;
 * n_subgraphs out (may be NULL).  Ties: lowest id.  A node that left the candidate set can still be
 * absorbed by a later candidate. */
ago_status ago_graph_cluster(int n_nodes, const double* weight, const unsigned char* is_complex,
                             int n_edges, const int* edge_src, const int* edge_dst, double td,
                             int max_complex, int* subgraph_of, int* n_subgraphs);

/* Split (Sec. V): Cluster applied inside every subgraph with threshold td_mini and at most one
 * complex operator per mini-subgraph.  mini_of:[n_nodes] out; parent_of_mini:[>= n_nodes] out, the
 * subgraph each mini-subgraph came from; n_minis out (may be NULL). */
ago_status ago_graph_split(int n_nodes, const double* weight, const unsigned char* is_complex, int n_edges,
                           const int* edge_src, const int* edge_dst, const int* subgraph_of, double td_mini,
                           int* mini_of, int* parent_of_mini, int* n_minis);

/* Join (Sec. V): the subgraph every node returns to when its mini-subgraphs are combined again. */
ago_status ago_graph_join(int n_nodes, const int* mini_of, int n_minis, const int* parent_of_mini,
                          int* subgraph_of);

/* Lowering (Sec. III-B, VI: the structures intensive fusion covers; Sec. III: sibling operators sharing an input):
 * inside every subgraph of a partition, recognise the operator chains the fused kernels implement and turn the
 * graph into a list of launches.  Host only.
 *
 * Graph: nodes 0..n_nodes-1 in topological order; op[v] is an ago_graph_op; the producers of node v are
 * input_ids[input_begin[v] .. input_begin[v+1]) (each < v, first operand first).  attr:[n_nodes][4] and
 * attr_f:[n_nodes] carry what the choice depends on (unused entries are ignored):
 *   DWCONV   attr[0] = stride                      CONV3X3  attr[0] = input channels
 *   GEMM     attr[0], attr[1] = rows, columns of its weight; attr[2] = rows of its input
 *   BMM_NT   attr[0] = last dimension of its first operand (the head dimension)
 *   TO_HEADS attr[0] = heads, attr[1] = 1 if the view is head-major ([B,Hh,S,D])
 *   SCALE    attr_f = the factor
 * subgraph_of:[n_nodes] is the partition (ago_graph_cluster).  dt is the storage type of the graph's tensors.
 * decide_ffn != 0: a matmul -> activation -> matmul chain becomes AGO_LAUNCH_FFN only where ago_fused_ffn_pays
 * says the fused kernel wins, else AGO_LAUNCH_FFN_EPILOGUE (two products with fused epilogues); 0: always fused.
 *
 * A chain starts at the first operator not yet placed and follows single-consumer links inside its subgraph (an
 * ADD may take its other operand from outside the chain, a batched product from anything computed before the
 * chain's start).  It is matched from its first operator against, in this order,
 *   INVRES      conv1x1 [bias] relu6 dwconv [bias] relu6 conv1x1 [bias] [add]   (add: the block's own input, stride 1)
 *   CONV_CHAIN  conv3x3 [bias] relu conv3x3 [bias] [add] relu                   (bf16, 64 channels)
 *   FFN         gemm [bias] (gelu_tanh | relu | relu6) gemm [bias]              (bf16)
 *   ATTN        bmm_nt scale softmax bmm_nn    (bf16, factor > 0, head dimension 64 or 128, the probabilities
 *                                               are the first operand of the second product)
 *   PW_DW       conv1x1 [bias] relu6 dwconv [bias] relu6
 *   DW_PW       dwconv [bias] relu6 conv1x1 [bias]
 * a structure whose residual is not admissible is retried without it.  QKV: three products that are the only
 * consumers of one tensor, in one subgraph, with equal weight shapes, each followed by [bias] and a TO_HEADS view
 * of equal form (bf16).  Everything else: AGO_LAUNCH_OP, one operator.  INPUT nodes launch nothing.
 *
 * Out: launch l has kind launch_kind[l] and the nodes launch_nodes[launch_begin[l] .. launch_begin[l+1]), chains in
 * chain order, QKV in increasing id; launches are in execution order.  launch_kind:[n_nodes],
 * launch_begin:[n_nodes+1], launch_nodes:[n_nodes], n_launches out.  Errors: NULL, SHAPE (ids out of range or not
 * topological, unknown operator), DTYPE. */
typedef enum { AGO_GOP_INPUT = 0, AGO_GOP_CONV1X1, AGO_GOP_DWCONV, AGO_GOP_CONV3X3, AGO_GOP_GEMM, AGO_GOP_BMM_NT,
               AGO_GOP_BMM_NN, AGO_GOP_BIAS, AGO_GOP_RELU, AGO_GOP_RELU6, AGO_GOP_GELU_TANH, AGO_GOP_ADD,
               AGO_GOP_SCALE, AGO_GOP_SOFTMAX, AGO_GOP_TO_HEADS, AGO_GOP_COUNT } ago_graph_op;
typedef enum { AGO_LAUNCH_OP = 0, AGO_LAUNCH_INVRES, AGO_LAUNCH_CONV_CHAIN, AGO_LAUNCH_FFN, AGO_LAUNCH_FFN_EPILOGUE,
               AGO_LAUNCH_ATTN, AGO_LAUNCH_PW_DW, AGO_LAUNCH_DW_PW, AGO_LAUNCH_QKV } ago_launch_kind;
ago_status ago_graph_lower(int n_nodes, const int* op, const int* input_begin, const int* input_ids,
                           const int* attr, const float* attr_f, const int* subgraph_of, ago_dtype dt,
                           int decide_ffn, int* launch_kind, int* launch_begin, int* launch_nodes, int* n_launches);

#ifdef __cplusplus
}
#endif
#endif /* AGO_H */
