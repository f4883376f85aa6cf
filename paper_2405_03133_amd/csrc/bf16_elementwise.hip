// SwiGLU forward and backward as streaming passes (HBM-bound).  Backward: from dA (left in the dG buffer by the
// dA = dY Wd_bar^T GEMM) and the saved G, U it produces, for one block of d_ff columns,
//   dG = dA * U * sig(G) * (1 + G (1 - sig(G))),  dU = dA * G * sig(G),  A = G sig(G) U
// (derivative of the LLaMA-style SwiGLU that the paper's experts use, Section 4.1).
#include "bf16_kernels.h"

namespace lory {
namespace k {

namespace {

__device__ __forceinline__ void unpack8(const uint4 &q, float (&f)[8])
{
    const uint32_t r[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(r[i] << 16);
        f[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
    }
}

__device__ __forceinline__ uint4 pack8(const float (&f)[8])
{
    uint4 q;
    q.x = gemm::cvt_pk_bf16(f[0], f[1]);
    q.y = gemm::cvt_pk_bf16(f[2], f[3]);
    q.z = gemm::cvt_pk_bf16(f[4], f[5]);
    q.w = gemm::cvt_pk_bf16(f[6], f[7]);
    return q;
}

// rows x (nf / 8) chunks of 8 columns; all arrays have row pitch dff and start at column n0.
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const uint16_t *__restrict__ G,
                                                         const uint16_t *__restrict__ U,
                                                         uint16_t *__restrict__ dG_dA,
                                                         uint16_t *__restrict__ dU,
                                                         uint16_t *__restrict__ Act, long rows, int dff,
                                                         int n0, int nf)
{
    const int cpr = nf >> 3;
    const long total = rows * cpr;
    for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (long)gridDim.x * blockDim.x) {
        const long row = idx / cpr;
        const int c = (int)(idx - row * cpr) << 3;
        const size_t off = (size_t)row * dff + n0 + c;
        float g[8], u[8], da[8], og[8], ou[8], oa[8];
        unpack8(*reinterpret_cast<const uint4 *>(G + off), g);
        unpack8(*reinterpret_cast<const uint4 *>(U + off), u);
        unpack8(*reinterpret_cast<const uint4 *>(dG_dA + off), da);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float sg = __builtin_amdgcn_rcpf(1.0f + __expf(-g[i]));
            oa[i] = g[i] * sg * u[i];
            og[i] = da[i] * u[i] * sg * (1.0f + g[i] * (1.0f - sg));
            ou[i] = da[i] * g[i] * sg;
        }
        *reinterpret_cast<uint4 *>(dG_dA + off) = pack8(og);
        *reinterpret_cast<uint4 *>(dU + off) = pack8(ou);
        *reinterpret_cast<uint4 *>(Act + off) = pack8(oa);
    }
}

// A = G * sigmoid(G) * U for one block of d_ff columns (SwiGLU forward, Section 4.1).
__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const uint16_t *__restrict__ G,
                                                         const uint16_t *__restrict__ U,
                                                         uint16_t *__restrict__ Act, long rows, int dff,
                                                         int n0, int nf)
{
    const int cpr = nf >> 3;
    const long total = rows * cpr;
    for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (long)gridDim.x * blockDim.x) {
        const long row = idx / cpr;
        const int c = (int)(idx - row * cpr) << 3;
        const size_t off = (size_t)row * dff + n0 + c;
        float g[8], u[8], oa[8];
        unpack8(*reinterpret_cast<const uint4 *>(G + off), g);
        unpack8(*reinterpret_cast<const uint4 *>(U + off), u);
#pragma unroll
        for (int i = 0; i < 8; ++i) oa[i] = g[i] * __builtin_amdgcn_rcpf(1.0f + __expf(-g[i])) * u[i];
        *reinterpret_cast<uint4 *>(Act + off) = pack8(oa);
    }
}

}  // namespace

hipError_t launch_swiglu_fwd(hipStream_t st, const uint16_t *G, const uint16_t *U, uint16_t *Act, long rows,
                             int dff, int n0, int nf)
{
    const long total = rows * (nf / 8);
    long blocks = (total + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(swiglu_fwd_kernel, dim3((unsigned)blocks), dim3(256), 0, st, G, U, Act, rows, dff, n0, nf);
    return hipGetLastError();
}

hipError_t launch_swiglu_bwd(hipStream_t st, const uint16_t *G, const uint16_t *U, uint16_t *dG_dA,
                             uint16_t *dU, uint16_t *Act, long rows, int dff, int n0, int nf)
{
    const long total = rows * (nf / 8);
    long blocks = (total + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(swiglu_bwd_kernel, dim3((unsigned)blocks), dim3(256), 0, st, G, U, dG_dA, dU, Act,
                       rows, dff, n0, nf);
    return hipGetLastError();
}

}  // namespace k
}  // namespace lory
