// Launch wrappers of the bf16 kernels; each group of instantiations lives in a
// translation unit of its own so that they compile in parallel.
#pragma once

#include "gemm_bf16.h"
#include "gemm2_bf16.h"
#include "merge_scatter_bf16.h"
#include "fused_bf16.h"
#include "fused_bwd_bf16.h"

namespace lory {
namespace k {

using gemm::bf16_bits_to_float;
using gemm::float_to_bf16_bits;

using gemm::u32x2;

struct NoIn {};

__device__ __forceinline__ u32x2 pack4(float a, float b, float c, float d)
{
    u32x2 r;
    r.x = gemm::cvt_pk_bf16(a, b);
    r.y = gemm::cvt_pk_bf16(c, d);
    return r;
}

__device__ __forceinline__ void unpack4(u32x2 p, float (&f)[4])
{
    f[0] = __uint_as_float(p.x << 16);
    f[1] = __uint_as_float(p.x & 0xffff0000u);
    f[2] = __uint_as_float(p.y << 16);
    f[3] = __uint_as_float(p.y & 0xffff0000u);
}

// Gate/up projections of one column block of d_ff: planes A = silu(G) * U, G, U.
// SAVE: write G and U; ACT: write A.  (Compile-time so that the epilogue has no data-dependent
// control flow.)
template <bool SAVE, bool ACT>
struct EpiGUT {
    static constexpr int NOUT = 3;
    // The ring GEMM forms the activation alone from the bf16 values of both operand sets
    // (combine) instead of calling pack() on the accumulators.
    static constexpr bool COMBINE = ACT && !SAVE;
    static constexpr int COMBINED_PLANE = 0;
    __device__ __forceinline__ gemm::u32x4 combine(gemm::u32x4 g, gemm::u32x4 u) const
    {
        gemm::u32x4 r;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float g0 = __uint_as_float(g[w] << 16), g1 = __uint_as_float(g[w] & 0xffff0000u);
            const float u0 = __uint_as_float(u[w] << 16), u1 = __uint_as_float(u[w] & 0xffff0000u);
            r[w] = gemm::cvt_pk_bf16(g0 * __builtin_amdgcn_rcpf(1.0f + __expf(-g0)) * u0,
                                     g1 * __builtin_amdgcn_rcpf(1.0f + __expf(-g1)) * u1);
        }
        return r;
    }
    static constexpr bool HAS_IN = false;
    typedef NoIn In;
    uint16_t *G, *U, *Act;  // [tokens, d_ff]
    int T, dff, n_off;
    __device__ __forceinline__ In load(int, int, int) const { return In(); }
    __device__ __forceinline__ bool enabled(int o) const { return o == 0 ? ACT : SAVE; }
    __device__ __forceinline__ u32x2 pack(int o, int, int, int, const In &, const float (&v)[2][4]) const
    {
        if (o == 1) return pack4(v[0][0], v[0][1], v[0][2], v[0][3]);
        if (o == 2) return pack4(v[1][0], v[1][1], v[1][2], v[1][3]);
        float a[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) a[e] = v[0][e] * __builtin_amdgcn_rcpf(1.0f + __expf(-v[0][e])) * v[1][e];
        return pack4(a[0], a[1], a[2], a[3]);
    }
    __device__ __forceinline__ uint16_t *ptr(int o, int s, int m, int n) const
    {
        uint16_t *base = (o == 0) ? Act : (o == 1) ? G : U;
        return base + ((size_t)s * T + m) * dff + n_off + n;
    }
};

// Run-time description of the same epilogue (G and U may both be NULL, Act may be NULL).
struct EpiGU {
    uint16_t *G, *U, *Act;
    int T, dff, n_off;
};

// C[batch][m][n] = bf16(v)
struct EpiStore {
    static constexpr int NOUT = 1;
    static constexpr bool COMBINE = false;
    static constexpr bool HAS_IN = false;
    typedef NoIn In;
    uint16_t *C;
    long c_batch;
    int ldc;
    __device__ __forceinline__ In load(int, int, int) const { return In(); }
    __device__ __forceinline__ bool enabled(int) const { return true; }
    __device__ __forceinline__ u32x2 pack(int, int, int, int, const In &, const float (&v)[1][4]) const
    {
        return pack4(v[0][0], v[0][1], v[0][2], v[0][3]);
    }
    __device__ __forceinline__ uint16_t *ptr(int, int b, int m, int n) const
    {
        return C + (size_t)b * c_batch + (size_t)m * ldc + n;
    }
};

struct EpiStore2 {
    static constexpr int NOUT = 2;
    static constexpr bool COMBINE = false;
    static constexpr bool HAS_IN = false;
    typedef NoIn In;
    uint16_t *C0, *C1;
    long c_batch;
    int ldc;
    __device__ __forceinline__ In load(int, int, int) const { return In(); }
    __device__ __forceinline__ bool enabled(int) const { return true; }
    __device__ __forceinline__ u32x2 pack(int o, int, int, int, const In &, const float (&v)[2][4]) const
    {
        return o == 0 ? pack4(v[0][0], v[0][1], v[0][2], v[0][3]) : pack4(v[1][0], v[1][1], v[1][2], v[1][3]);
    }
    __device__ __forceinline__ uint16_t *ptr(int o, int b, int m, int n) const
    {
        return (o == 0 ? C0 : C1) + (size_t)b * c_batch + (size_t)m * ldc + n;
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

// merge inside the GEMM (fused_bf16.h): C = sum over nsrc sources of A_q * Wbar_q(segment of the row)
bool fused_fits(const fmg::Params &p);
hipError_t launch_fused(hipStream_t st, const fmg::Params &p, int nsrc, bool w_nc);

// expert gradients and routing-weight inner products with the per-segment weight gradients kept on
// chip (fused_bwd_bf16.h); the partial-sum buffer holds fused_dw_slots(p) x S x 16 floats
bool fused_dw_fits(const fsg::Params &p);
int fused_dw_slots(const fsg::Params &p);
hipError_t launch_fused_dw(hipStream_t st, const fsg::Params &p);

hipError_t launch_gu(hipStream_t st, const gemm::Params &p, const EpiGU &e);     // X * [Wg_bar | Wu_bar]
hipError_t launch_down(hipStream_t st, const gemm::Params &p, const EpiStore &e);  // A * Wd_bar
hipError_t launch_da(hipStream_t st, const gemm::Params &p, const EpiStore &e);  // dY * Wd_bar^T
hipError_t launch_swiglu_fwd(hipStream_t st, const uint16_t *G, const uint16_t *U, uint16_t *Act, long rows,
                             int dff, int n0, int nf);
hipError_t launch_swiglu_bwd(hipStream_t st, const uint16_t *G, const uint16_t *U, uint16_t *dG_dA,
                             uint16_t *dU, uint16_t *Act, long rows, int dff, int n0, int nf);
hipError_t launch_dx(hipStream_t st, const gemm::Params &p, const EpiStore &e);  // dG Wg_bar^T + dU Wu_bar^T
hipError_t launch_dwgu(hipStream_t st, const gemm::Params &p, const EpiStore2 &e);  // X^T [dG | dU]
hipError_t launch_dwd(hipStream_t st, const gemm::Params &p, const EpiStore &e);  // A^T dY

}  // namespace k
}  // namespace lory
