/*
 * CPU oracle for chains of dependent tiled kernels (test infrastructure only).
 *
 * Fine-grained synchronisation changes only WHEN a consumer tile may start
 * (Section III of the paper: kernels on separate streams, per-tile
 * semaphores); it never changes WHAT is computed.  The result of a chain is
 * therefore the plain definition of the two (or three) operators applied one
 * after the other, and that definition is what this file writes out:
 *
 *   MLP chain          (Fig. 2a)  Y = GeLU(X W1) W2
 *   gated MLP chain    (Fig. 3)   Y = (silu(X Wg) * (X Wu)) W2
 *   attention chain    (Fig. 2b)  Y = causal_attention(X Wqkv) Wo
 *   Conv2D chain       (Sec. IV-B "Conv2D", Table II)  two 3x3 convolutions,
 *                      stride 1, zero padding 1, ReLU between them
 *
 * Everything is fp64, naive loops, no tiling, no fusion.  The only
 * parallelism is an OpenMP "parallel for" over independent output rows or
 * pixels, which does not change any summation order.  Nothing here is shared
 * with, included by, or linked into the GPU library; only tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.
 *
 * All matrices are dense row-major.  A weight matrix W of a product X W is
 * passed in its mathematical shape [K x N].
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- pointwise operators ------------------------------------------------ */

/* GeLU, exact form x * Phi(x) with the normal CDF Phi written through erf. */
double oracle_gelu(double x) { return 0.5 * x * (1.0 + erf(x / sqrt(2.0))); }

/* Swish with beta = 1 (SiLU): x * sigmoid(x). */
double oracle_silu(double x) { return x / (1.0 + exp(-x)); }

double oracle_relu(double x) { return x > 0.0 ? x : 0.0; }

enum { ORACLE_ACT_NONE = 0, ORACLE_ACT_GELU = 1, ORACLE_ACT_RELU = 2 };

static double apply_act(int act, double x) {
    switch (act) {
        case ORACLE_ACT_GELU: return oracle_gelu(x);
        case ORACLE_ACT_RELU: return oracle_relu(x);
        default: return x;
    }
}

/* ---- GeMM --------------------------------------------------------------- */

/* C[M x N] = A[M x K] B[K x N]; every C[i][j] sums k = 0..K-1 in order. */
void oracle_gemm(long M, long N, long K, const double* A, const double* B, double* C) {
#pragma omp parallel for schedule(static)
    for (long i = 0; i < M; ++i) {
        double* c = C + i * N;
        for (long j = 0; j < N; ++j) c[j] = 0.0;
        for (long k = 0; k < K; ++k) {
            const double a = A[i * K + k];
            const double* b = B + k * N;
            for (long j = 0; j < N; ++j) c[j] += a * b[j];
        }
    }
}

void oracle_act_inplace(long n, int act, double* x) {
#pragma omp parallel for schedule(static)
    for (long i = 0; i < n; ++i) x[i] = apply_act(act, x[i]);
}

/*
 * MLP chain (Fig. 2a): H = act(X W1), Y = H W2.
 * X[M x K1], W1[K1 x N1], W2[N1 x N2]; H[M x N1] and Y[M x N2] are outputs.
 */
void oracle_gemm_chain(long M, long K1, long N1, long N2, const double* X, const double* W1,
                       const double* W2, int act, double* H, double* Y) {
    oracle_gemm(M, N1, K1, X, W1, H);
    oracle_act_inplace(M * N1, act, H);
    oracle_gemm(M, N2, N1, H, W2, Y);
}

/*
 * Gated MLP chain (Fig. 3, with the first two GeMMs combined into one weight
 * matrix as Section II-B describes): Wgu[K1 x 2*Nh] holds the gate weights in
 * columns [0, Nh) and the up weights in columns [Nh, 2*Nh).
 *   G = X Wgate, U = X Wup, H = silu(G) * U (elementwise), Y = H W2.
 * GU[M x 2*Nh] (scratch/output), H[M x Nh], Y[M x N2].
 */
void oracle_swiglu_chain(long M, long K1, long Nh, long N2, const double* X, const double* Wgu,
                         const double* W2, double* GU, double* H, double* Y) {
    oracle_gemm(M, 2 * Nh, K1, X, Wgu, GU);
#pragma omp parallel for schedule(static)
    for (long i = 0; i < M; ++i)
        for (long j = 0; j < Nh; ++j)
            H[i * Nh + j] = oracle_silu(GU[i * 2 * Nh + j]) * GU[i * 2 * Nh + Nh + j];
    oracle_gemm(M, N2, Nh, H, W2, Y);
}

/* ---- causal attention --------------------------------------------------- */

/*
 * Per-head causal attention on the output of the QKV GeMM (Fig. 2b, prompt
 * phase: no cached keys or values, dropout is the identity at inference).
 * QKV[M x ldq] with M = batch*seq rows; query, key and value of head h sit in
 * columns qoff + h*d, koff + h*d, voff + h*d (d wide each).
 * For batch b, head h, query row i:  p_j = q_i . k_j / sqrt(d) for j <= i,
 * r = softmax(p), t_i = sum_j r_j v_j.  T[M x ldt], head h in columns h*d.
 * Only heads [h0, h1) are computed.
 */
void oracle_causal_attention(long batch, long seq, long heads, long d, const double* QKV,
                             long ldq, long qoff, long koff, long voff, double* T, long ldt,
                             long h0, long h1) {
    (void)heads;
    const double scale = 1.0 / sqrt((double)d);
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
    for (long b = 0; b < batch; ++b) {
        for (long i = 0; i < seq; ++i) {
            double* p = (double*)malloc((size_t)(i + 1) * sizeof(double));
            for (long h = h0; h < h1; ++h) {
                const double* q = QKV + (b * seq + i) * ldq + qoff + h * d;
                double mx = -INFINITY;
                for (long j = 0; j <= i; ++j) {
                    const double* k = QKV + (b * seq + j) * ldq + koff + h * d;
                    double s = 0.0;
                    for (long e = 0; e < d; ++e) s += q[e] * k[e];
                    p[j] = s * scale;
                    if (p[j] > mx) mx = p[j];
                }
                double den = 0.0;
                for (long j = 0; j <= i; ++j) {
                    p[j] = exp(p[j] - mx);
                    den += p[j];
                }
                double* t = T + (b * seq + i) * ldt + h * d;
                for (long e = 0; e < d; ++e) t[e] = 0.0;
                for (long j = 0; j <= i; ++j) {
                    const double r = p[j] / den;
                    const double* v = QKV + (b * seq + j) * ldq + voff + h * d;
                    for (long e = 0; e < d; ++e) t[e] += r * v[e];
                }
            }
            free(p);
        }
    }
}

/*
 * Attention chain (Fig. 2b): QKV = X Wqkv; T = per-head causal attention;
 * Y = T Wo.  Column layout of QKV: Q block, then K block, then V block, each
 * heads*d wide.  X[M x K1], Wqkv[K1 x 3*heads*d], Wo[heads*d x N2].
 */
void oracle_attn_chain(long batch, long seq, long heads, long d, long K1, long N2,
                       const double* X, const double* Wqkv, const double* Wo, double* QKV,
                       double* T, double* Y) {
    const long M = batch * seq, E = heads * d;
    oracle_gemm(M, 3 * E, K1, X, Wqkv, QKV);
    oracle_causal_attention(batch, seq, heads, d, QKV, 3 * E, 0, E, 2 * E, T, E, 0, heads);
    oracle_gemm(M, N2, E, T, Wo, Y);
}

/* ---- Conv2D ------------------------------------------------------------- */

/*
 * 3x3 (generally R x S) cross-correlation, stride 1, zero padding (R-1)/2,
 * NHWC activations, weights [K][R][S][C]:
 *   out[b,y,x,k] = act( sum_{r,s,c} in[b, y+r-pr, x+s-ps, c] * w[k,r,s,c] )
 * with terms whose input coordinate falls outside the image left out.
 */
void oracle_conv2d_nhwc(long B, long H, long W, long C, long K, long R, long S,
                        const double* in, const double* w, int act, double* out) {
    const long pr = (R - 1) / 2, ps = (S - 1) / 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (long b = 0; b < B; ++b) {
        for (long y = 0; y < H; ++y) {
            for (long x = 0; x < W; ++x) {
                for (long k = 0; k < K; ++k) {
                    double acc = 0.0;
                    for (long r = 0; r < R; ++r) {
                        const long yy = y + r - pr;
                        if (yy < 0 || yy >= H) continue;
                        for (long s = 0; s < S; ++s) {
                            const long xx = x + s - ps;
                            if (xx < 0 || xx >= W) continue;
                            const double* ip = in + ((b * H + yy) * W + xx) * C;
                            const double* wp = w + ((k * R + r) * S + s) * C;
                            for (long c = 0; c < C; ++c) acc += ip[c] * wp[c];
                        }
                    }
                    out[((b * H + y) * W + x) * K + k] = apply_act(act, acc);
                }
            }
        }
    }
}

/* Conv chain: mid = relu(conv(in, w1)); out = conv(mid, w2). */
void oracle_conv_chain(long B, long H, long W, long C, long K1, long K2, const double* in,
                       const double* w1, const double* w2, double* mid, double* out) {
    oracle_conv2d_nhwc(B, H, W, C, K1, 3, 3, in, w1, ORACLE_ACT_RELU, mid);
    oracle_conv2d_nhwc(B, H, W, K1, K2, 3, 3, mid, w2, ORACLE_ACT_NONE, out);
}

/*
 * The same chain evaluated only at n sampled output pixels (b,y,x triples in
 * pix[3*i..]): out_s[n x K2].  Each output pixel depends on a 3x3
 * neighbourhood of mid, i.e. a 5x5 neighbourhood of the input; the needed mid
 * values are computed from the definition on the fly.
 */
void oracle_conv_chain_pixels(long B, long H, long W, long C, long K1, long K2,
                              const double* in, const double* w1, const double* w2, long n,
                              const long* pix, double* out_s) {
    (void)B;
#pragma omp parallel for schedule(dynamic, 1)
    for (long i = 0; i < n; ++i) {
        const long b = pix[3 * i], y = pix[3 * i + 1], x = pix[3 * i + 2];
        double* mid = (double*)calloc((size_t)(9 * K1), sizeof(double));
        char have[9];
        for (long r = 0; r < 3; ++r)
            for (long s = 0; s < 3; ++s) {
                const long my = y + r - 1, mx = x + s - 1;
                have[r * 3 + s] = (my >= 0 && my < H && mx >= 0 && mx < W);
                if (!have[r * 3 + s]) continue;
                for (long k = 0; k < K1; ++k) {
                    double acc = 0.0;
                    for (long r1 = 0; r1 < 3; ++r1) {
                        const long yy = my + r1 - 1;
                        if (yy < 0 || yy >= H) continue;
                        for (long s1 = 0; s1 < 3; ++s1) {
                            const long xx = mx + s1 - 1;
                            if (xx < 0 || xx >= W) continue;
                            const double* ip = in + ((b * H + yy) * W + xx) * C;
                            const double* wp = w1 + ((k * 3 + r1) * 3 + s1) * C;
                            for (long c = 0; c < C; ++c) acc += ip[c] * wp[c];
                        }
                    }
                    mid[(r * 3 + s) * K1 + k] = oracle_relu(acc);
                }
            }
        for (long k2 = 0; k2 < K2; ++k2) {
            double acc = 0.0;
            for (long r = 0; r < 3; ++r)
                for (long s = 0; s < 3; ++s) {
                    if (!have[r * 3 + s]) continue;
                    const double* mp = mid + (r * 3 + s) * K1;
                    const double* wp = w2 + ((k2 * 3 + r) * 3 + s) * K1;
                    for (long k = 0; k < K1; ++k) acc += mp[k] * wp[k];
                }
            out_s[i * K2 + k2] = acc;
        }
        free(mid);
    }
}
