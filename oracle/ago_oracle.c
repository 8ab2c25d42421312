/*
 * CPU oracle for fused multi-complex-operator subgraphs (TEST INFRASTRUCTURE).
 *
 * This file is test infrastructure, not product code: only the tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it.  It shares no
 * code, header, table or helper with the HIP library.
 *
 * Everything is evaluated operator by operator in fp64 on dense arrays with
 * full-size intermediates, exactly as the paper's un-fused loop nest does
 * (Sec. III-A, Fig. 3: one nest for the convolution, one for the bias, one
 * for the ReLU).  Fusion, conventional (Fig. 4) or intensive (Sec. III-B,
 * Fig. 5), is only a re-ordering of these loops and must give the same
 * tensor, so the plain definition is the reference for every fused kernel.
 *
 * Conventions (the paper writes NCHW / OIHW; the benchmark fixes NHWC):
 *   activations  [N][H][W][C], C fastest
 *   1x1 weights  [Cin][Cout]          3x3 weights [3][3][Cin][Cout]
 *   depthwise    [3][3][C]            GEMM operands row-major
 * Convolution is cross-correlation (Fig. 3: Inp[h+rr][w+rc]*Weight[rr][rc],
 * no kernel flip).  Spatial padding is zero padding of the operator's *input
 * tensor*; for the second operator of a chain that is the post-activation
 * intermediate.
 *
 * OpenMP only parallelises the outermost independent loop; the summation
 * order of every output element is the textual order of the definition.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ---- complex operators -------------------------------------------------- */

/* Pointwise convolution == matrix product over the channel axis (Sec. III-B:
 * no reduction over the window, R = C = 1).  y[p][o] = sum_c x[p][c] w[c][o] */
void ago_oracle_conv1x1(const double* x, const double* w, double* y,
                        long P, int Cin, int Cout) {
#pragma omp parallel for schedule(static)
    for (long p = 0; p < P; ++p) {
        double* yp = y + p * Cout;
        for (int o = 0; o < Cout; ++o) yp[o] = 0.0;
        for (int c = 0; c < Cin; ++c) {
            const double xv = x[p * Cin + c];
            const double* wr = w + (long)c * Cout;
            for (int o = 0; o < Cout; ++o) yp[o] += xv * wr[o];
        }
    }
}

/* Row-major matrix product c[M][N] = a[M][K] b[K][N]. */
void ago_oracle_gemm(const double* a, const double* b, double* c, int M, int K, int N) {
    ago_oracle_conv1x1(a, b, c, (long)M, K, N);
}

/* Depthwise 3x3, zero pad 1, stride st: no reduction over channels.
 * y[n][oh][ow][c] = sum_{r,s} xpad[n][oh*st + r - 1][ow*st + s - 1][c] w[r][s][c] */
void ago_oracle_dwconv3x3(const double* x, const double* w, double* y,
                          int N, int H, int W, int C, int st) {
    const int OH = (H + 2 - 3) / st + 1, OW = (W + 2 - 3) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int oh = 0; oh < OH; ++oh)
            for (int ow = 0; ow < OW; ++ow) {
                double* yp = y + (((long)n * OH + oh) * OW + ow) * C;
                for (int c = 0; c < C; ++c) {
                    double acc = 0.0;
                    for (int r = 0; r < 3; ++r)
                        for (int s = 0; s < 3; ++s) {
                            const int ih = oh * st + r - 1, iw = ow * st + s - 1;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue; /* zero pad */
                            acc += x[(((long)n * H + ih) * W + iw) * C + c] * w[(r * 3 + s) * C + c];
                        }
                    yp[c] = acc;
                }
            }
}

/* Depthwise R x R for odd R (the 5x5 depthwise layers of the MNasNet-style blocks among the paper's
 * mobile networks, Sec. VI), zero pad (R-1)/2, stride st:
 * y[n][oh][ow][c] = sum_{r,s} xpad[n][oh*st + r - pad][ow*st + s - pad][c] w[r][s][c] */
void ago_oracle_dwconv(const double* x, const double* w, double* y,
                       int N, int H, int W, int C, int st, int R) {
    const int pad = (R - 1) / 2;
    const int OH = (H + 2 * pad - R) / st + 1, OW = (W + 2 * pad - R) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int oh = 0; oh < OH; ++oh)
            for (int ow = 0; ow < OW; ++ow)
                for (int c = 0; c < C; ++c) {
                    double acc = 0.0;
                    for (int r = 0; r < R; ++r)
                        for (int s = 0; s < R; ++s) {
                            const int ih = oh * st + r - pad, iw = ow * st + s - pad;
                            if (ih >= 0 && ih < H && iw >= 0 && iw < W)
                                acc += x[(((long)n * H + ih) * W + iw) * C + c] * w[((long)r * R + s) * C + c];
                        }
                    y[(((long)n * OH + oh) * OW + ow) * C + c] = acc;
                }
}

/* Dense 3x3 convolution, zero pad 1, stride 1 (Fig. 3 with R = C = 3).
 * y[n][h][w][o] = sum_{r,s,c} xpad[n][h+r-1][w+s-1][c] wt[r][s][c][o] */
void ago_oracle_conv3x3(const double* x, const double* wt, double* y,
                        int N, int H, int W, int Cin, int Cout) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int h = 0; h < H; ++h)
            for (int w = 0; w < W; ++w) {
                double* yp = y + (((long)n * H + h) * W + w) * Cout;
                for (int o = 0; o < Cout; ++o) yp[o] = 0.0;
                for (int r = 0; r < 3; ++r)
                    for (int s = 0; s < 3; ++s) {
                        const int ih = h + r - 1, iw = w + s - 1;
                        if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;   /* zero pad */
                        const double* xp = x + (((long)n * H + ih) * W + iw) * Cin;
                        for (int c = 0; c < Cin; ++c) {
                            const double xv = xp[c];
                            const double* wr = wt + ((long)((r * 3 + s) * Cin + c)) * Cout;
                            for (int o = 0; o < Cout; ++o) yp[o] += xv * wr[o];
                        }
                    }
            }
}

/* Batched a[b] (S x D) times transpose of k[b] (S2 x D): s[b][i][j] = sum_d a[i][d] k[j][d]. */
void ago_oracle_bmm_nt(const double* a, const double* k, double* s,
                       long batch, int S, int S2, int D) {
#pragma omp parallel for collapse(2) schedule(static)
    for (long b = 0; b < batch; ++b)
        for (int i = 0; i < S; ++i) {
            const double* ai = a + (b * S + i) * D;
            for (int j = 0; j < S2; ++j) {
                const double* kj = k + (b * S2 + j) * D;
                double acc = 0.0;
                for (int d = 0; d < D; ++d) acc += ai[d] * kj[d];
                s[(b * S + i) * S2 + j] = acc;
            }
        }
}

/* Batched p[b] (S x S2) times v[b] (S2 x D). */
void ago_oracle_bmm_nn(const double* p, const double* v, double* o,
                       long batch, int S, int S2, int D) {
#pragma omp parallel for schedule(static)
    for (long b = 0; b < batch; ++b)
        ago_oracle_conv1x1(p + b * S * S2, v + b * S2 * D, o + b * S * D, S, S2, D);
}

/* ---- simple operators (each its own pass, as in Fig. 3) ------------------ */

void ago_oracle_bias(double* y, const double* b, long P, int C) {
#pragma omp parallel for schedule(static)
    for (long p = 0; p < P; ++p)
        for (int c = 0; c < C; ++c) y[p * C + c] += b[c];
}

void ago_oracle_relu(double* y, long n) {
#pragma omp parallel for schedule(static)
    for (long i = 0; i < n; ++i) y[i] = y[i] > 0.0 ? y[i] : 0.0;
}

void ago_oracle_relu6(double* y, long n) {
#pragma omp parallel for schedule(static)
    for (long i = 0; i < n; ++i) {
        double v = y[i] > 0.0 ? y[i] : 0.0;
        y[i] = v < 6.0 ? v : 6.0;
    }
}

/* GELU, tanh form: 0.5 x (1 + tanh( sqrt(2/pi) (x + 0.044715 x^3) )). */
void ago_oracle_gelu_tanh(double* y, long n) {
    const double k = 0.79788456080286535588; /* sqrt(2/pi) */
#pragma omp parallel for schedule(static)
    for (long i = 0; i < n; ++i) {
        const double x = y[i];
        y[i] = 0.5 * x * (1.0 + tanh(k * (x + 0.044715 * x * x * x)));
    }
}

void ago_oracle_add(double* y, const double* x, long n) {
#pragma omp parallel for schedule(static)
    for (long i = 0; i < n; ++i) y[i] += x[i];
}

void ago_oracle_scale(double* y, double a, long n) {
#pragma omp parallel for schedule(static)
    for (long i = 0; i < n; ++i) y[i] *= a;
}

/* Row softmax with the row maximum subtracted first. */
void ago_oracle_softmax_rows(double* s, long rows, int cols) {
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        double* p = s + r * cols;
        double m = p[0];
        for (int j = 1; j < cols; ++j) if (p[j] > m) m = p[j];
        double sum = 0.0;
        for (int j = 0; j < cols; ++j) { p[j] = exp(p[j] - m); sum += p[j]; }
        for (int j = 0; j < cols; ++j) p[j] /= sum;
    }
}

/* ---- the four subgraphs, operator by operator ---------------------------- */

static double* dalloc(long n) { return (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1)); }

/* pointwise expand -> depthwise -> pointwise project (MobileNetV2-style block:
 * the pw->dw and dw->pw pairs of Sec. III-B, Fig. 7).  Returns 0, or -1 on
 * allocation failure.  Biases may be NULL. */
int ago_oracle_invres(const double* x, const double* w1, const double* b1,
                      const double* wd, const double* bd,
                      const double* w2, const double* b2, double* y,
                      int N, int H, int W, int Cin, int Cexp, int Cout,
                      int stride, int residual) {
    const int OH = (H + 2 - 3) / stride + 1, OW = (W + 2 - 3) / stride + 1;
    const long PE = (long)N * H * W, PO = (long)N * OH * OW;
    double* e = dalloc(PE * Cexp);
    double* d = dalloc(PO * Cexp);
    if (!e || !d) { free(e); free(d); return -1; }
    ago_oracle_conv1x1(x, w1, e, PE, Cin, Cexp);
    if (b1) ago_oracle_bias(e, b1, PE, Cexp);
    ago_oracle_relu6(e, PE * Cexp);
    ago_oracle_dwconv3x3(e, wd, d, N, H, W, Cexp, stride);
    if (bd) ago_oracle_bias(d, bd, PO, Cexp);
    ago_oracle_relu6(d, PO * Cexp);
    ago_oracle_conv1x1(d, w2, y, PO, Cexp, Cout);
    if (b2) ago_oracle_bias(y, b2, PO, Cout);
    if (residual) ago_oracle_add(y, x, PO * Cout);
    free(e); free(d);
    return 0;
}

/* conv3x3 + bias + ReLU -> conv3x3 + bias (+ x) -> ReLU (the general-conv
 * downstream case of Sec. III-B, Fig. 5, with zero padding). */
int ago_oracle_conv_chain(const double* x, const double* wa, const double* ba,
                          const double* wb, const double* bb, double* y,
                          int N, int H, int W, int C, int residual) {
    const long P = (long)N * H * W;
    double* t = dalloc(P * C);
    if (!t) return -1;
    ago_oracle_conv3x3(x, wa, t, N, H, W, C, C);
    if (ba) ago_oracle_bias(t, ba, P, C);
    ago_oracle_relu(t, P * C);
    ago_oracle_conv3x3(t, wb, y, N, H, W, C, C);
    if (bb) ago_oracle_bias(y, bb, P, C);
    if (residual) ago_oracle_add(y, x, P * C);
    ago_oracle_relu(y, P * C);
    free(t);
    return 0;
}

/* GEMM + bias + GELU -> GEMM + bias (pw->pw; a matrix product is a pointwise
 * convolution, Sec. III-B).  act: 0 none, 1 relu, 2 relu6, 3 gelu_tanh. */
int ago_oracle_ffn(const double* x, const double* w1, const double* b1,
                   const double* w2, const double* b2, double* y,
                   int M, int K, int F, int K2, int act) {
    double* h = dalloc((long)M * F);
    if (!h) return -1;
    ago_oracle_gemm(x, w1, h, M, K, F);
    if (b1) ago_oracle_bias(h, b1, M, F);
    if (act == 1) ago_oracle_relu(h, (long)M * F);
    else if (act == 2) ago_oracle_relu6(h, (long)M * F);
    else if (act == 3) ago_oracle_gelu_tanh(h, (long)M * F);
    ago_oracle_gemm(h, w2, y, M, F, K2);
    if (b2) ago_oracle_bias(y, b2, M, K2);
    free(h);
    return 0;
}

/* matmul -> scale -> row softmax -> matmul per (batch, head). */
int ago_oracle_attn(const double* q, const double* k, const double* v, double* o,
                    int B, int Hh, int S, int D, double scale) {
    const long batch = (long)B * Hh;
    double* s = dalloc(batch * S * S);
    if (!s) return -1;
    ago_oracle_bmm_nt(q, k, s, batch, S, S, D);
    ago_oracle_scale(s, scale, batch * S * S);
    ago_oracle_softmax_rows(s, batch * S, S);
    ago_oracle_bmm_nn(s, v, o, batch, S, S, D);
    free(s);
    return 0;
}
