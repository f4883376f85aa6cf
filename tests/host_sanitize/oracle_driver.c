/* Runs every function of the CPU oracle on small problems with exactly sized heap buffers, for a
 * build with -fsanitize=address,undefined: any out-of-bounds access, use of uninitialised
 * bookkeeping or undefined arithmetic in the oracle aborts the run.  Prints checksums. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

int lory_oracle_route(long B, long L, long T, long d, long E, const double *X, const double *R, double *hbar,
                      double *e, double *w);
int lory_oracle_ffn_fwd(long S, long T, long d, long dff, long E, const double *X, const double *w, const double *Wg,
                        const double *Wu, const double *Wd, double *Y, double *G_out, double *U_out);
int lory_oracle_ffn_bwd(long S, long T, long d, long dff, long E, const double *X, const double *w, const double *Wg,
                        const double *Wu, const double *Wd, const double *dY, double *dX, double *dWg, double *dWu,
                        double *dWd, double *dw);
int lory_oracle_route_bwd(long B, long L, long T, long d, long E, const double *X, const double *R, const double *dw,
                          double *dX_add, double *dR);

static unsigned long long state = 88172645463325252ULL;
static double rnd(void)
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0 - 0.5;
}
static double *fill(long n, double scale)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)n);
    for (long i = 0; i < n; ++i) p[i] = scale * rnd();
    return p;
}
static double sum(const double *p, long n)
{
    double s = 0.0;
    for (long i = 0; i < n; ++i) s += p[i];
    return s;
}

static int run(long B, long L, long T, long d, long dff, long E)
{
    const long N = L / T, S = B * N, D = d * dff;
    double *X = fill(B * L * d, 2.0), *R = fill(d * E, 0.5), *dY = fill(B * L * d, 2.0);
    double *Wg = fill(E * D, 0.1), *Wu = fill(E * D, 0.1), *Wd = fill(E * D, 0.1);
    double *hbar = fill(S * d, 0), *e = fill(S * E, 0), *w = fill(S * E, 0);
    double *Y = fill(B * L * d, 0), *G = fill(B * L * dff, 0), *U = fill(B * L * dff, 0);
    double *dX = fill(B * L * d, 0), *dWg = fill(E * D, 0), *dWu = fill(E * D, 0), *dWd = fill(E * D, 0);
    double *dw = fill(S * E, 0), *dXa = fill(B * L * d, 0), *dR = fill(d * E, 0);
    int rc = 0;
    rc |= lory_oracle_route(B, L, T, d, E, X, R, hbar, e, w);
    rc |= lory_oracle_ffn_fwd(S, T, d, dff, E, X, w, Wg, Wu, Wd, Y, G, U);
    rc |= lory_oracle_ffn_fwd(S, T, d, dff, E, X, w, Wg, Wu, Wd, Y, NULL, NULL);
    rc |= lory_oracle_ffn_bwd(S, T, d, dff, E, X, w, Wg, Wu, Wd, dY, dX, dWg, dWu, dWd, dw);
    rc |= lory_oracle_route_bwd(B, L, T, d, E, X, R, dw, dXa, dR);
    printf("B=%ld L=%ld T=%ld d=%ld dff=%ld E=%ld rc=%d  w=%.6f Y=%.6e dX=%.6e dW=%.6e dw=%.6e dR=%.6e\n", B, L, T, d,
           dff, E, rc, sum(w, S * E), sum(Y, B * L * d), sum(dX, B * L * d),
           sum(dWg, E * D) + sum(dWu, E * D) + sum(dWd, E * D), sum(dw, S * E), sum(dR, d * E));
    if (fabs(sum(w, S * E) - (double)S) > 1e-9) rc |= 2; /* rows of w sum to one */
    free(X); free(R); free(dY); free(Wg); free(Wu); free(Wd); free(hbar); free(e); free(w); free(Y); free(G);
    free(U); free(dX); free(dWg); free(dWu); free(dWd); free(dw); free(dXa); free(dR);
    return rc;
}

int main(void)
{
    int rc = 0;
    rc |= run(2, 12, 4, 5, 7, 3);    /* ragged everything */
    rc |= run(1, 8, 8, 16, 24, 1);   /* one segment, one expert */
    rc |= run(3, 6, 1, 3, 2, 64);    /* one-token segments, many experts */
    rc |= run(2, 64, 16, 32, 48, 8);
    /* a ragged tail is refused, nothing is written */
    double dummy = 0.0;
    if (lory_oracle_route(1, 10, 4, 2, 2, &dummy, &dummy, &dummy, &dummy, &dummy) == 0) rc |= 4;
    printf("oracle sanitizer run: %s\n", rc ? "FAILED" : "ok");
    return rc;
}
