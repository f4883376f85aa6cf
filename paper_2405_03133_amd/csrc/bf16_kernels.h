// Launch wrappers of the bf16 kernels; each group of instantiations lives in a
// translation unit of its own so that they compile in parallel.
#pragma once

#include "gemm_bf16.h"
#include "merge_scatter_bf16.h"

namespace lory {
namespace k {

using gemm::bf16_bits_to_float;
using gemm::float_to_bf16_bits;

// G, U (optional) and A = silu(G) * U of one column block of d_ff.
struct EpiGU {
    uint16_t *G, *U, *Act;  // [tokens, d_ff]; G and U may both be NULL
    int T, dff, n_off;
    __device__ __forceinline__ void operator()(int s, int m, int n, const float (&v)[2]) const
    {
        const size_t idx = ((size_t)s * T + m) * dff + n_off + n;
        const float g = v[0], u = v[1];
        if (G) {
            G[idx] = float_to_bf16_bits(g);
            U[idx] = float_to_bf16_bits(u);
        }
        if (Act) Act[idx] = float_to_bf16_bits(g / (1.0f + __expf(-g)) * u);
    }
};

// C[batch][m][n] = bf16(v)
struct EpiStore {
    uint16_t *C;
    long c_batch;
    int ldc;
    __device__ __forceinline__ void operator()(int b, int m, int n, const float (&v)[1]) const
    {
        C[(size_t)b * c_batch + (size_t)m * ldc + n] = float_to_bf16_bits(v[0]);
    }
};

struct EpiStore2 {
    uint16_t *C0, *C1;
    long c_batch;
    int ldc;
    __device__ __forceinline__ void operator()(int b, int m, int n, const float (&v)[2]) const
    {
        const size_t idx = (size_t)b * c_batch + (size_t)m * ldc + n;
        C0[idx] = float_to_bf16_bits(v[0]);
        C1[idx] = float_to_bf16_bits(v[1]);
    }
};

// SwiGLU backward fused behind dA = dY Wd_bar^T:
//   dG = dA * U * sig(G) * (1 + G (1 - sig(G))),  dU = dA * G * sig(G),  A = G sig(G) U
struct EpiDA {
    const uint16_t *G, *U;       // saved forward activations [tokens, d_ff]
    uint16_t *dG, *dU, *Act;     // [tokens, d_ff]
    int T, dff, n_off;
    __device__ __forceinline__ void operator()(int s, int m, int n, const float (&v)[1]) const
    {
        const size_t idx = ((size_t)s * T + m) * dff + n_off + n;
        const float g = bf16_bits_to_float(G[idx]), u = bf16_bits_to_float(U[idx]);
        const float da = v[0];
        const float sg = 1.0f / (1.0f + __expf(-g));
        Act[idx] = float_to_bf16_bits(g * sg * u);
        dG[idx] = float_to_bf16_bits(da * u * sg * (1.0f + g * (1.0f - sg)));
        dU[idx] = float_to_bf16_bits(da * g * sg);
    }
};

// Every wrapper returns a hipError_t.  M, N, K must be multiples of the tile
// sizes the wrapper picks (64 granularity is always accepted).
hipError_t launch_merge(hipStream_t st, const ms::MergeParams &p);
hipError_t launch_scatter(hipStream_t st, const ms::ScatterParams &p, int grid);
hipError_t launch_dw_reduce(hipStream_t st, const float *partials, int slots, int rows, int cols,
                            float *dw, int S, int E);
int scatter_grid();                       // workgroups the scatter kernel is launched with
void scatter_partial_dims(int S, int E, int *rows, int *cols);

hipError_t launch_gu(hipStream_t st, const gemm::Params &p, const EpiGU &e);     // X * [Wg_bar | Wu_bar]
hipError_t launch_down(hipStream_t st, const gemm::Params &p, const EpiStore &e);  // A * Wd_bar
hipError_t launch_da(hipStream_t st, const gemm::Params &p, const EpiDA &e);     // dY * Wd_bar^T
hipError_t launch_dx(hipStream_t st, const gemm::Params &p, const EpiStore &e);  // dG Wg_bar^T + dU Wu_bar^T
hipError_t launch_dwgu(hipStream_t st, const gemm::Params &p, const EpiStore2 &e);  // X^T [dG | dU]
hipError_t launch_dwd(hipStream_t st, const gemm::Params &p, const EpiStore &e);  // A^T dY

}  // namespace k
}  // namespace lory
