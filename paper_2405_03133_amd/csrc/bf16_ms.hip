// Instantiations of the merge / scatter / router-weight-gradient kernels.
#include "bf16_kernels.h"

namespace lory {
namespace k {

namespace {
// dw[s][e] = sum over slots of partials[slot][s][e].  One workgroup per segment row: thread
// (e, g) adds slots g, g+16, ... along four interleaved chains (fixed order), then the 16 group
// sums are added in order.
__global__ __launch_bounds__(1024) void dw_reduce_kernel(const float *__restrict__ partials, int slots,
                                                         int rows, int cols, float *__restrict__ dw,
                                                         int S, int E)
{
    __shared__ float red[16][64];
    const int s = blockIdx.x;
    const int e = threadIdx.x & 63, g = threadIdx.x >> 6;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    if (e < E) {
        const float *src = partials + (size_t)s * cols + e;
        const size_t pitch = (size_t)rows * cols;
        int k = g;
        for (; k + 48 < slots; k += 64) {
            a0 += src[(size_t)k * pitch];
            a1 += src[(size_t)(k + 16) * pitch];
            a2 += src[(size_t)(k + 32) * pitch];
            a3 += src[(size_t)(k + 48) * pitch];
        }
        for (; k < slots; k += 16) a0 += src[(size_t)k * pitch];
    }
    red[g][e] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    if (g == 0 && e < E) {
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) sum += red[i][e];
        dw[(size_t)s * E + e] = sum;
    }
}

constexpr int kMsGrid = 1024;  // workgroups; 4 wavefronts each stride over the 256-element units

int units_of(const ms::Rect &rc) { return ((rc.nr * rc.nc / 8) + 31) / 32; }
}  // namespace

int scatter_grid() { return kMsGrid; }

namespace {
int kbm_of(int S)
{
    const int KB = (S + 15) / 16;
    int kbm = 1;
    while (kbm < KB) kbm *= 2;
    return kbm;
}
}  // namespace

void scatter_partial_dims(int S, int E, int *rows, int *cols)
{
    *rows = kbm_of(S) * 16;
    *cols = ((E + 31) / 32) * 32;
}

hipError_t launch_merge(hipStream_t st, const ms::MergeParams &p)
{
    const int KS = (p.E + 15) / 16;
    const int MB = (p.S + 31) / 32;
    const size_t lds = (size_t)MB * KS * 2 * 64 * 16;
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    int grid = (units_of(p.rc) + 3) / 4;
    if (grid > kMsGrid) grid = kMsGrid;
    switch (KS) {
    case 1: hipLaunchKernelGGL(ms::merge_kernel<1>, dim3(grid), dim3(256), lds, st, p); break;
    case 2: hipLaunchKernelGGL(ms::merge_kernel<2>, dim3(grid), dim3(256), lds, st, p); break;
    case 3: hipLaunchKernelGGL(ms::merge_kernel<3>, dim3(grid), dim3(256), lds, st, p); break;
    case 4: hipLaunchKernelGGL(ms::merge_kernel<4>, dim3(grid), dim3(256), lds, st, p); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_scatter(hipStream_t st, const ms::ScatterParams &p, int grid)
{
    const int KB = (p.S + 15) / 16;
    if (KB > 16 || p.e0 % 32 != 0 || p.e0 >= p.E) return hipErrorInvalidValue;
    const int win = (p.E - p.e0 < 32) ? (p.E - p.e0) : 32;
    const int eb16 = (win + 15) / 16;
    const size_t lds_main = (size_t)KB * 2 * 64 * 16 + 4 * 16 * ms::kDotPitch;
#define LORY_SCATTER(K, B)                                                                            \
    do {                                                                                              \
        const size_t lds_red = (size_t)4 * K * B * 1024;                                              \
        const size_t lds_work = lds_main + (ms::scatter_parks_experts<K, B>() ? 4 * B * 4096 : 0);    \
        const size_t lds = lds_work > lds_red ? lds_work : lds_red;                                   \
        auto kern = ms::scatter_kernel<K, B>;                                                         \
        if (lds > 48 * 1024) {                                                                        \
            static bool configured = false;                                                           \
            if (!configured) {                                                                        \
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),              \
                                                   hipFuncAttributeMaxDynamicSharedMemorySize,        \
                                                   160 * 1024);                                       \
                if (e != hipSuccess) return e;                                                        \
                configured = true;                                                                    \
            }                                                                                         \
        }                                                                                             \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, p);                                  \
    } while (0)
#define LORY_SCATTER_K(B)                          \
    switch (kbm_of(p.S)) {                         \
    case 1: LORY_SCATTER(1, B); break;             \
    case 2: LORY_SCATTER(2, B); break;             \
    case 4: LORY_SCATTER(4, B); break;             \
    case 8: LORY_SCATTER(8, B); break;             \
    default: LORY_SCATTER(16, B); break;           \
    }
    if (eb16 == 1) {
        LORY_SCATTER_K(1)
    } else {
        LORY_SCATTER_K(2)
    }
#undef LORY_SCATTER_K
#undef LORY_SCATTER
    return hipGetLastError();
}

hipError_t launch_dw_reduce(hipStream_t st, const float *partials, int slots, int rows, int cols,
                            float *dw, int S, int E)
{
    hipLaunchKernelGGL(dw_reduce_kernel, dim3(S), dim3(1024), 0, st, partials, slots, rows, cols, dw, S,
                       E);
    return hipGetLastError();
}

}  // namespace k
}  // namespace lory
