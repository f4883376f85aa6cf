/*
 * CPU fp64 oracle for the Lory causal-segment expert-merging MoE FFN layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP
 * library is checked against; the product never calls it.  It shares no code
 * with the HIP path.
 *
 * The method is exact (a re-association of a plain definition, not an
 * approximation), so the oracle evaluates that definition literally:
 *   - segment mean, linear router, softmax          (Section 3.1, Eq. 2)
 *   - causal shift with the first-segment rule      (Section 3.1; Algorithm 1)
 *   - parameter-space merge  theta_bar = sum_i e_i * theta_i   (Eq. 1, Eq. 2)
 *   - LLaMA-style SwiGLU FFN with the merged parameters applied to every
 *     token of the segment                          (Section 3.1; Section 4.1)
 *   - backward: chain rule on the above, written out by hand.
 * Merged weights are fully materialised per segment; every floating-point
 * operation is in double.  Loops are the textbook triple loops (i-k-j order);
 * OpenMP only splits the outermost independent loop.
 *
 * Conventions: all arrays are row-major, last index fastest.
 *   X  [S*T, d]     hidden states, S = B*(L/T) segments of T tokens
 *   R  [d, E]       router, no bias
 *   Wg, Wu [E, d, d_ff]; Wd [E, d_ff, d]
 *   w  [S, E]       routing weights actually used by segment s
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

/* C[M,N] = A[M,K] * B[K,N] */
static void mm_nn(long M, long N, long K, const double *A, const double *B, double *C)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < M; ++i) {
        double *c = C + i * N;
        for (long j = 0; j < N; ++j) c[j] = 0.0;
        for (long k = 0; k < K; ++k) {
            const double a = A[i * K + k];
            const double *b = B + k * N;
            for (long j = 0; j < N; ++j) c[j] += a * b[j];
        }
    }
}

/* C[M,N] = A[M,K] * B[N,K]^T */
static void mm_nt(long M, long N, long K, const double *A, const double *B, double *C)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < M; ++i) {
        for (long j = 0; j < N; ++j) {
            double acc = 0.0;
            for (long k = 0; k < K; ++k) acc += A[i * K + k] * B[j * K + k];
            C[i * N + j] = acc;
        }
    }
}

/* C[M,N] = A[K,M]^T * B[K,N] */
static void mm_tn(long M, long N, long K, const double *A, const double *B, double *C)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < M; ++i) {
        double *c = C + i * N;
        for (long j = 0; j < N; ++j) c[j] = 0.0;
        for (long k = 0; k < K; ++k) {
            const double a = A[k * M + i];
            const double *b = B + k * N;
            for (long j = 0; j < N; ++j) c[j] += a * b[j];
        }
    }
}

static double sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }

/* theta_bar = sum_e w[e] * theta_e  for one matrix of n elements (Eq. 2). */
static void merge_one(long E, long n, const double *w_row, const double *stack, double *merged)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < n; ++i) {
        double acc = 0.0;
        for (long e = 0; e < E; ++e) acc += w_row[e] * stack[e * n + i];
        merged[i] = acc;
    }
}

/*
 * Routing (Section 3.1, Eq. 2; Algorithm 1).
 *   hbar[b,k,:] = mean over the T tokens of segment k of sequence b
 *   e[b,k,:]    = softmax(hbar[b,k,:] * R)
 *   w[b,0,:]    = e[b,0,:]          (first segment routes on itself)
 *   w[b,k,:]    = e[b,k-1,:], k>=1  (causal shift by one segment)
 * Outputs hbar [B*N,d], e [B*N,E], w [B*N,E].  Returns nonzero if L % T != 0.
 */
int lory_oracle_route(long B, long L, long T, long d, long E,
                      const double *X, const double *R,
                      double *hbar, double *e, double *w)
{
    if (T <= 0 || L % T != 0) return 1;
    const long N = L / T;
    double *z = (double *)malloc(sizeof(double) * (size_t)E);
    for (long b = 0; b < B; ++b) {
        for (long k = 0; k < N; ++k) {
            double *h = hbar + (b * N + k) * d;
            for (long j = 0; j < d; ++j) h[j] = 0.0;
            for (long t = 0; t < T; ++t) {
                const double *x = X + ((b * L) + k * T + t) * d;
                for (long j = 0; j < d; ++j) h[j] += x[j];
            }
            for (long j = 0; j < d; ++j) h[j] /= (double)T;
            double zmax = -INFINITY;
            for (long i = 0; i < E; ++i) {
                double acc = 0.0;
                for (long j = 0; j < d; ++j) acc += h[j] * R[j * E + i];
                z[i] = acc;
                if (acc > zmax) zmax = acc;
            }
            double denom = 0.0;
            for (long i = 0; i < E; ++i) { z[i] = exp(z[i] - zmax); denom += z[i]; }
            for (long i = 0; i < E; ++i) e[(b * N + k) * E + i] = z[i] / denom;
        }
        for (long k = 0; k < N; ++k) {
            const long src = (k == 0) ? 0 : k - 1;
            for (long i = 0; i < E; ++i) w[(b * N + k) * E + i] = e[(b * N + src) * E + i];
        }
    }
    free(z);
    return 0;
}

/*
 * Merged FFN forward (Eq. 1 / Eq. 2 with the SwiGLU FFN of Section 4.1):
 * for every segment s, merge the three matrices with w[s,:] and compute
 *   G = X_s Wg_bar,  U = X_s Wu_bar,  A = G*sigmoid(G) (.) U,  Y_s = A Wd_bar.
 * G_out, U_out (each [S*T, d_ff]) may be NULL.
 */
int lory_oracle_ffn_fwd(long S, long T, long d, long dff, long E,
                        const double *X, const double *w,
                        const double *Wg, const double *Wu, const double *Wd,
                        double *Y, double *G_out, double *U_out)
{
    const long D = d * dff;
    double *mg = (double *)malloc(sizeof(double) * (size_t)D);
    double *mu = (double *)malloc(sizeof(double) * (size_t)D);
    double *md = (double *)malloc(sizeof(double) * (size_t)D);
    double *G = (double *)malloc(sizeof(double) * (size_t)(T * dff));
    double *U = (double *)malloc(sizeof(double) * (size_t)(T * dff));
    double *A = (double *)malloc(sizeof(double) * (size_t)(T * dff));
    if (!mg || !mu || !md || !G || !U || !A) return 2;
    for (long s = 0; s < S; ++s) {
        const double *Xs = X + s * T * d;
        merge_one(E, D, w + s * E, Wg, mg);
        merge_one(E, D, w + s * E, Wu, mu);
        merge_one(E, D, w + s * E, Wd, md);
        mm_nn(T, dff, d, Xs, mg, G);
        mm_nn(T, dff, d, Xs, mu, U);
        for (long i = 0; i < T * dff; ++i) A[i] = G[i] * sigmoid(G[i]) * U[i];
        mm_nn(T, d, dff, A, md, Y + s * T * d);
        if (G_out) memcpy(G_out + s * T * dff, G, sizeof(double) * (size_t)(T * dff));
        if (U_out) memcpy(U_out + s * T * dff, U, sizeof(double) * (size_t)(T * dff));
    }
    free(mg); free(mu); free(md); free(G); free(U); free(A);
    return 0;
}

/*
 * Merged FFN backward with w treated as an independent input.  Given dY:
 *   dA  = dY Wd_bar^T            dWd_bar = A^T dY
 *   dG  = dA (.) U (.) sig(G) (1 + G (1 - sig(G)))      dU = dA (.) G sig(G)
 *   dWg_bar = X^T dG             dWu_bar = X^T dU
 *   dX  = dG Wg_bar^T + dU Wu_bar^T
 *   dWx[e] += w[s,e] * dWx_bar   dw[s,e] = sum_x <Wx[e], dWx_bar>
 * (chain rule on theta_bar = sum_i e_i theta_i, Eq. 2).  dWg, dWu, dWd are
 * overwritten (zeroed first).  dw is returned for all segments; a stop
 * gradient on the first segment is the router backward's business.
 */
int lory_oracle_ffn_bwd(long S, long T, long d, long dff, long E,
                        const double *X, const double *w,
                        const double *Wg, const double *Wu, const double *Wd,
                        const double *dY,
                        double *dX, double *dWg, double *dWu, double *dWd, double *dw)
{
    const long D = d * dff;
    const long TF = T * dff;
    double *mg = (double *)malloc(sizeof(double) * (size_t)D);
    double *mu = (double *)malloc(sizeof(double) * (size_t)D);
    double *md = (double *)malloc(sizeof(double) * (size_t)D);
    double *gg = (double *)malloc(sizeof(double) * (size_t)D);
    double *gu = (double *)malloc(sizeof(double) * (size_t)D);
    double *gd = (double *)malloc(sizeof(double) * (size_t)D);
    double *G = (double *)malloc(sizeof(double) * (size_t)TF);
    double *U = (double *)malloc(sizeof(double) * (size_t)TF);
    double *A = (double *)malloc(sizeof(double) * (size_t)TF);
    double *dA = (double *)malloc(sizeof(double) * (size_t)TF);
    double *dG = (double *)malloc(sizeof(double) * (size_t)TF);
    double *dU = (double *)malloc(sizeof(double) * (size_t)TF);
    double *t1 = (double *)malloc(sizeof(double) * (size_t)(T * d));
    double *t2 = (double *)malloc(sizeof(double) * (size_t)(T * d));
    if (!mg || !mu || !md || !gg || !gu || !gd || !G || !U || !A || !dA || !dG || !dU || !t1 || !t2) return 2;
    memset(dWg, 0, sizeof(double) * (size_t)(E * D));
    memset(dWu, 0, sizeof(double) * (size_t)(E * D));
    memset(dWd, 0, sizeof(double) * (size_t)(E * D));
    for (long s = 0; s < S; ++s) {
        const double *Xs = X + s * T * d;
        const double *dYs = dY + s * T * d;
        const double *ws = w + s * E;
        merge_one(E, D, ws, Wg, mg);
        merge_one(E, D, ws, Wu, mu);
        merge_one(E, D, ws, Wd, md);
        mm_nn(T, dff, d, Xs, mg, G);
        mm_nn(T, dff, d, Xs, mu, U);
        for (long i = 0; i < TF; ++i) A[i] = G[i] * sigmoid(G[i]) * U[i];
        mm_nt(T, dff, d, dYs, md, dA);      /* dA = dY Wd_bar^T */
        mm_tn(dff, d, T, A, dYs, gd);       /* dWd_bar = A^T dY */
        for (long i = 0; i < TF; ++i) {
            const double sg = sigmoid(G[i]);
            dG[i] = dA[i] * U[i] * sg * (1.0 + G[i] * (1.0 - sg));
            dU[i] = dA[i] * G[i] * sg;
        }
        mm_tn(d, dff, T, Xs, dG, gg);       /* dWg_bar = X^T dG */
        mm_tn(d, dff, T, Xs, dU, gu);       /* dWu_bar = X^T dU */
        mm_nt(T, d, dff, dG, mg, t1);       /* dG Wg_bar^T */
        mm_nt(T, d, dff, dU, mu, t2);       /* dU Wu_bar^T */
        for (long i = 0; i < T * d; ++i) dX[s * T * d + i] = t1[i] + t2[i];
        for (long e = 0; e < E; ++e) {
            const double we = ws[e];
            double dot = 0.0;
            const double *a = Wg + e * D, *b = Wu + e * D, *c = Wd + e * D;
            double *ga = dWg + e * D, *gb = dWu + e * D, *gc = dWd + e * D;
#pragma omp parallel for schedule(static) reduction(+ : dot)
            for (long i = 0; i < D; ++i) {
                ga[i] += we * gg[i];
                gb[i] += we * gu[i];
                gc[i] += we * gd[i];
                dot += a[i] * gg[i] + b[i] * gu[i] + c[i] * gd[i];
            }
            dw[s * E + e] = dot;
        }
    }
    free(mg); free(mu); free(md); free(gg); free(gu); free(gd);
    free(G); free(U); free(A); free(dA); free(dG); free(dU); free(t1); free(t2);
    return 0;
}

/*
 * Router backward for the whole layer (Section 3.1; Algorithm 1): takes the
 * dw [B*N,E] that lory_oracle_ffn_bwd produced and pushes it through the
 * first-segment stop gradient, the causal shift, the softmax, the linear
 * router and the segment mean.
 *   dw[b,0,:] is dropped (stop gradient on the first segment's routing);
 *   de[b,j,:] = dw[b,j+1,:] for j < N-1, de[b,N-1,:] = 0;
 *   dz = e (.) (de - <e,de>);  dR += hbar^T dz;  dhbar = dz R^T;
 *   dX_add[b, jT+t, :] = dhbar[b,j,:] / T.
 * dX_add [B*L,d] and dR [d,E] are overwritten.
 */
int lory_oracle_route_bwd(long B, long L, long T, long d, long E,
                          const double *X, const double *R, const double *dw,
                          double *dX_add, double *dR)
{
    if (T <= 0 || L % T != 0) return 1;
    const long N = L / T;
    const long S = B * N;
    double *hbar = (double *)malloc(sizeof(double) * (size_t)(S * d));
    double *e = (double *)malloc(sizeof(double) * (size_t)(S * E));
    double *w = (double *)malloc(sizeof(double) * (size_t)(S * E));
    double *de = (double *)malloc(sizeof(double) * (size_t)E);
    double *dz = (double *)malloc(sizeof(double) * (size_t)E);
    if (!hbar || !e || !w || !de || !dz) return 2;
    lory_oracle_route(B, L, T, d, E, X, R, hbar, e, w);
    for (long i = 0; i < d * E; ++i) dR[i] = 0.0;
    for (long b = 0; b < B; ++b) {
        for (long j = 0; j < N; ++j) {
            const long s = b * N + j;
            for (long i = 0; i < E; ++i) de[i] = (j < N - 1) ? dw[(s + 1) * E + i] : 0.0;
            double inner = 0.0;
            for (long i = 0; i < E; ++i) inner += e[s * E + i] * de[i];
            for (long i = 0; i < E; ++i) dz[i] = e[s * E + i] * (de[i] - inner);
            for (long c = 0; c < d; ++c) {
                double acc = 0.0;
                for (long i = 0; i < E; ++i) {
                    dR[c * E + i] += hbar[s * d + c] * dz[i];
                    acc += dz[i] * R[c * E + i];
                }
                for (long t = 0; t < T; ++t) dX_add[(b * L + j * T + t) * d + c] = acc / (double)T;
            }
        }
    }
    free(hbar); free(e); free(w); free(de); free(dz);
    return 0;
}
