// fp32 instantiation of the merged FFN (paper Eq. 1 / Eq. 2, SwiGLU experts)
// and of its backward.  This path exists for the small fp32 configuration
// whose tolerance (rel-L2 <= 1e-5) needs fp32 operands; it is written for
// clarity and arbitrary shapes, not for speed: LDS-tiled FMA GEMMs, explicit
// per-segment merged weights in a workspace slab, processed a chunk of
// segments at a time so that the workspace stays bounded.
#include "lory_internal.h"

namespace lory {

namespace {

constexpr size_t kF32ChunkBudget = (size_t)512 << 20;  // workspace target per chunk of segments

// ---------------------------------------------------------------- kernels

// slab[s][i] = sum_e w[s][e] * stack[e][i]      grid (ceil(n/256), Sc)
__global__ void merge_f32_kernel(const float *__restrict__ w, const float *__restrict__ stack,
                                 float *__restrict__ slab, long n, int E)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int s = blockIdx.y;
    if (i >= n) return;
    float acc = 0.f;
    for (int e = 0; e < E; ++e) acc = fmaf(w[(size_t)s * E + e], stack[(size_t)e * n + i], acc);
    slab[(size_t)s * n + i] = acc;
}

// Batched C = op(A) * op(B) (+ C), 64x64x16 tiles, 256 threads, 4x4 per thread.
//   op(A)(m,k) = TA ? A[k*lda + m] : A[m*lda + k]
//   op(B)(k,n) = TB ? B[n*ldb + k] : B[k*ldb + n]
template <bool TA, bool TB>
__global__ __launch_bounds__(256) void sgemm_kernel(int M, int N, int K, const float *__restrict__ A,
                                                    int lda, long strideA,
                                                    const float *__restrict__ B, int ldb,
                                                    long strideB, float *__restrict__ C, int ldc,
                                                    long strideC, int add)
{
    __shared__ float As[16][64 + 4];
    __shared__ float Bs[16][64 + 4];
    A += (size_t)blockIdx.z * strideA;
    B += (size_t)blockIdx.z * strideB;
    C += (size_t)blockIdx.z * strideC;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int tid = threadIdx.x;
    const int tm = (tid / 16) * 4, tn = (tid % 16) * 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int i = tid; i < 64 * 16; i += 256) {
            int mm, kk;
            if (TA) { mm = i % 64; kk = i / 64; } else { kk = i % 16; mm = i / 16; }
            const int gm = m0 + mm, gk = k0 + kk;
            float v = 0.f;
            if (gm < M && gk < K) v = TA ? A[(size_t)gk * lda + gm] : A[(size_t)gm * lda + gk];
            As[kk][mm] = v;
        }
        for (int i = tid; i < 64 * 16; i += 256) {
            int nn, kk;
            if (TB) { kk = i % 16; nn = i / 16; } else { nn = i % 64; kk = i / 64; }
            const int gn = n0 + nn, gk = k0 + kk;
            float v = 0.f;
            if (gn < N && gk < K) v = TB ? B[(size_t)gn * ldb + gk] : B[(size_t)gk * ldb + gn];
            Bs[kk][nn] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][tm + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tn + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    for (int i = 0; i < 4; ++i) {
        const int gm = m0 + tm + i;
        if (gm >= M) continue;
        for (int j = 0; j < 4; ++j) {
            const int gn = n0 + tn + j;
            if (gn >= N) continue;
            float *c = C + (size_t)gm * ldc + gn;
            *c = add ? (*c + acc[i][j]) : acc[i][j];
        }
    }
}

__device__ inline float sigmoidf_(float z) { return 1.0f / (1.0f + expf(-z)); }

// A = G * sigmoid(G) * U
__global__ void swiglu_fwd_kernel(const float *__restrict__ G, const float *__restrict__ U,
                                  float *__restrict__ A, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float g = G[i];
    A[i] = g * sigmoidf_(g) * U[i];
}

// dG = dA * U * sig(G) * (1 + G (1 - sig(G))),  dU = dA * G * sig(G); also A (needed for dWd_bar)
__global__ void swiglu_bwd_kernel(const float *__restrict__ G, const float *__restrict__ U,
                                  const float *__restrict__ dA, float *__restrict__ A,
                                  float *__restrict__ dG, float *__restrict__ dU, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float g = G[i], u = U[i], da = dA[i];
    const float sg = sigmoidf_(g);
    A[i] = g * sg * u;
    dG[i] = da * u * sg * (1.0f + g * (1.0f - sg));
    dU[i] = da * g * sg;
}

// dW[e][i] (+)= sum_{s in chunk} w[s][e] * slab[s][i]      grid (ceil(n/256), E)
__global__ void scatter_f32_kernel(const float *__restrict__ w, const float *__restrict__ slab,
                                   float *__restrict__ dW, long n, int E, int Sc, int add)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int e = blockIdx.y;
    if (i >= n) return;
    float acc = 0.f;
    for (int s = 0; s < Sc; ++s) acc = fmaf(w[(size_t)s * E + e], slab[(size_t)s * n + i], acc);
    float *p = dW + (size_t)e * n + i;
    *p = add ? (*p + acc) : acc;
}

// dw[s][e] (+)= <stack[e], slab[s]>      grid (E, Sc), 256 threads, fixed-order tree reduction
__global__ __launch_bounds__(256) void dots_f32_kernel(const float *__restrict__ stack,
                                                       const float *__restrict__ slab,
                                                       float *__restrict__ dw, long n, int E, int add)
{
    __shared__ float red[256];
    const int e = blockIdx.x, s = blockIdx.y;
    const float *a = stack + (size_t)e * n;
    const float *b = slab + (size_t)s * n;
    float acc = 0.f;
    for (long i = threadIdx.x; i < n; i += 256) acc = fmaf(a[i], b[i], acc);
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        float *p = dw + (size_t)s * E + e;
        *p = add ? (*p + red[0]) : red[0];
    }
}

// ---------------------------------------------------------------- host helpers

struct F32Plan {
    int Sc;           // segments per chunk
    size_t slab;      // floats of one merged (or gradient) slab: Sc * D
    size_t act;       // floats of one activation buffer: Sc * T * d_ff
};

F32Plan plan(const Dims &m)
{
    const size_t per_seg = (size_t)4 * (6 * (size_t)m.D + 6 * (size_t)m.T * m.dff);
    long sc = (long)(kF32ChunkBudget / per_seg);
    if (sc < 1) sc = 1;
    if (sc > m.S) sc = m.S;
    F32Plan p;
    p.Sc = (int)sc;
    p.slab = (size_t)p.Sc * m.D;
    p.act = (size_t)p.Sc * m.T * m.dff;
    return p;
}

template <bool TA, bool TB>
void gemm(hipStream_t st, int batch, int M, int N, int K, const float *A, int lda, long sA,
          const float *B, int ldb, long sB, float *C, int ldc, long sC, int add)
{
    const dim3 grid((N + 63) / 64, (M + 63) / 64, batch);
    hipLaunchKernelGGL((sgemm_kernel<TA, TB>), grid, dim3(256), 0, st, M, N, K, A, lda, sA, B, ldb,
                       sB, C, ldc, sC, add);
}

void merge(hipStream_t st, const float *w, const float *stack, float *slab, long n, int E, int Sc)
{
    const dim3 grid((unsigned)((n + 255) / 256), Sc);
    hipLaunchKernelGGL(merge_f32_kernel, grid, dim3(256), 0, st, w, stack, slab, n, E);
}

}  // namespace

size_t f32_workspace_bytes(const Dims &m, int pass)
{
    const F32Plan p = plan(m);
    if (pass == LORY_PASS_FWD) return sizeof(float) * (3 * p.slab + 3 * p.act);
    return sizeof(float) * (6 * p.slab + 6 * p.act);
}

int f32_ffn_fwd(const Dims &m, const float *X, const float *w, const float *Wg, const float *Wu,
                const float *Wd, float *Y, float *G_save, float *U_save, void *ws, hipStream_t st)
{
    const F32Plan p = plan(m);
    float *mg = (float *)ws, *mu = mg + p.slab, *md = mu + p.slab;
    float *Gb = md + p.slab, *Ub = Gb + p.act, *Ab = Ub + p.act;
    const long TD = (long)m.T * m.d, TF = (long)m.T * m.dff;
    for (int s0 = 0; s0 < m.S; s0 += p.Sc) {
        const int sc = (m.S - s0 < p.Sc) ? (m.S - s0) : p.Sc;
        const float *wc = w + (size_t)s0 * m.E;
        const float *Xc = X + (size_t)s0 * TD;
        float *G = G_save ? G_save + (size_t)s0 * TF : Gb;
        float *U = U_save ? U_save + (size_t)s0 * TF : Ub;
        merge(st, wc, Wg, mg, m.D, m.E, sc);
        merge(st, wc, Wu, mu, m.D, m.E, sc);
        merge(st, wc, Wd, md, m.D, m.E, sc);
        gemm<false, false>(st, sc, m.T, m.dff, m.d, Xc, m.d, TD, mg, m.dff, m.D, G, m.dff, TF, 0);
        gemm<false, false>(st, sc, m.T, m.dff, m.d, Xc, m.d, TD, mu, m.dff, m.D, U, m.dff, TF, 0);
        const long n = (long)sc * TF;
        hipLaunchKernelGGL(swiglu_fwd_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, G,
                           U, Ab, n);
        gemm<false, false>(st, sc, m.T, m.d, m.dff, Ab, m.dff, TF, md, m.d, m.D,
                           Y + (size_t)s0 * TD, m.d, TD, 0);
    }
    return launch_status();
}

// Merged parameters of all m.S segments as [Wg_bar | Wu_bar | Wd_bar], each [S][rows][cols].
int f32_merge_all(const Dims &m, const float *w, const float *Wg, const float *Wu, const float *Wd,
                  float *Wbar, hipStream_t st)
{
    const float *stacks[3] = {Wg, Wu, Wd};
    for (int x = 0; x < 3; ++x)
        for (int s0 = 0; s0 < m.S; s0 += 32768) {  // grid.y limit
            const int sc = (m.S - s0 < 32768) ? (m.S - s0) : 32768;
            merge(st, w + (size_t)s0 * m.E, stacks[x], Wbar + ((size_t)x * m.S + s0) * m.D, m.D, m.E, sc);
        }
    return launch_status();
}

int f32_ffn_bwd(const Dims &m, const float *X, const float *w, const float *Wg, const float *Wu,
                const float *Wd, const float *dY, const float *G_save, const float *U_save,
                float *dX, float *dWg, float *dWu, float *dWd, int accumulate, float *dw, void *ws,
                hipStream_t st)
{
    const F32Plan p = plan(m);
    float *mg = (float *)ws, *mu = mg + p.slab, *md = mu + p.slab;
    float *gg = md + p.slab, *gu = gg + p.slab, *gd = gu + p.slab;
    float *Gb = gd + p.slab, *Ub = Gb + p.act, *Ab = Ub + p.act;
    float *dAb = Ab + p.act, *dGb = dAb + p.act, *dUb = dGb + p.act;
    const long TD = (long)m.T * m.d, TF = (long)m.T * m.dff;
    for (int s0 = 0; s0 < m.S; s0 += p.Sc) {
        const int sc = (m.S - s0 < p.Sc) ? (m.S - s0) : p.Sc;
        const float *wc = w + (size_t)s0 * m.E;
        const float *Xc = X + (size_t)s0 * TD;
        const float *dYc = dY + (size_t)s0 * TD;
        merge(st, wc, Wg, mg, m.D, m.E, sc);
        merge(st, wc, Wu, mu, m.D, m.E, sc);
        merge(st, wc, Wd, md, m.D, m.E, sc);
        const float *G, *U;
        if (G_save && U_save) {
            G = G_save + (size_t)s0 * TF;
            U = U_save + (size_t)s0 * TF;
        } else {
            gemm<false, false>(st, sc, m.T, m.dff, m.d, Xc, m.d, TD, mg, m.dff, m.D, Gb, m.dff, TF, 0);
            gemm<false, false>(st, sc, m.T, m.dff, m.d, Xc, m.d, TD, mu, m.dff, m.D, Ub, m.dff, TF, 0);
            G = Gb;
            U = Ub;
        }
        // dA = dY Wd_bar^T
        gemm<false, true>(st, sc, m.T, m.dff, m.d, dYc, m.d, TD, md, m.d, m.D, dAb, m.dff, TF, 0);
        const long n = (long)sc * TF;
        hipLaunchKernelGGL(swiglu_bwd_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, G,
                           U, dAb, Ab, dGb, dUb, n);
        // dWd_bar = A^T dY ; dWg_bar = X^T dG ; dWu_bar = X^T dU
        gemm<true, false>(st, sc, m.dff, m.d, m.T, Ab, m.dff, TF, dYc, m.d, TD, gd, m.d, m.D, 0);
        gemm<true, false>(st, sc, m.d, m.dff, m.T, Xc, m.d, TD, dGb, m.dff, TF, gg, m.dff, m.D, 0);
        gemm<true, false>(st, sc, m.d, m.dff, m.T, Xc, m.d, TD, dUb, m.dff, TF, gu, m.dff, m.D, 0);
        // dX = dG Wg_bar^T + dU Wu_bar^T
        float *dXc = dX + (size_t)s0 * TD;
        gemm<false, true>(st, sc, m.T, m.d, m.dff, dGb, m.dff, TF, mg, m.dff, m.D, dXc, m.d, TD, 0);
        gemm<false, true>(st, sc, m.T, m.d, m.dff, dUb, m.dff, TF, mu, m.dff, m.D, dXc, m.d, TD, 1);
        // scatter to the experts and router-weight inner products
        const int add = (accumulate || s0 > 0) ? 1 : 0;
        const dim3 sgrid((unsigned)((m.D + 255) / 256), m.E);
        hipLaunchKernelGGL(scatter_f32_kernel, sgrid, dim3(256), 0, st, wc, gg, dWg, m.D, m.E, sc, add);
        hipLaunchKernelGGL(scatter_f32_kernel, sgrid, dim3(256), 0, st, wc, gu, dWu, m.D, m.E, sc, add);
        hipLaunchKernelGGL(scatter_f32_kernel, sgrid, dim3(256), 0, st, wc, gd, dWd, m.D, m.E, sc, add);
        float *dwc = dw + (size_t)s0 * m.E;
        const dim3 dgrid(m.E, sc);
        hipLaunchKernelGGL(dots_f32_kernel, dgrid, dim3(256), 0, st, Wg, gg, dwc, m.D, m.E, 0);
        hipLaunchKernelGGL(dots_f32_kernel, dgrid, dim3(256), 0, st, Wu, gu, dwc, m.D, m.E, 1);
        hipLaunchKernelGGL(dots_f32_kernel, dgrid, dim3(256), 0, st, Wd, gd, dwc, m.D, m.E, 1);
    }
    return launch_status();
}

}  // namespace lory
