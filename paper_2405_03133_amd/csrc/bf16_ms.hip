// Instantiations of the merge / scatter / router-weight-gradient kernels.
#include "bf16_kernels.h"

namespace lory {
namespace k {

namespace {
// dw[s][e] = sum over slots of partials[slot][s][e], in slot order.
__global__ void dw_reduce_kernel(const float *__restrict__ partials, int slots, int rows, int cols,
                                 float *__restrict__ dw, int S, int E)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= S * E) return;
    const int s = idx / E, e = idx % E;
    float acc = 0.f;
    for (int k = 0; k < slots; ++k) acc += partials[((size_t)k * rows + s) * cols + e];
    dw[idx] = acc;
}


constexpr int kMsGrid = 1024;  // workgroups; 4 wavefronts each stride over the 256-element units

int units_of(const ms::Rect &rc) { return ((rc.nr * rc.nc / 8) + 31) / 32; }
}  // namespace

int scatter_grid() { return kMsGrid; }

void scatter_partial_dims(int S, int E, int *rows, int *cols)
{
    const int SB = (S + 31) / 32, EB = (E + 31) / 32;
    int nacc = 1;
    while (nacc < SB * EB) nacc *= 2;
    *rows = (nacc / EB) * 32;
    *cols = EB * 32;
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
    const int SB = (p.S + 31) / 32, EB = (p.E + 31) / 32, KB = (p.S + 15) / 16;
    const size_t lds = (size_t)EB * KB * 2 * 64 * 16;
    if (lds > 64 * 1024 || SB * EB > 8 || EB > 2) return hipErrorInvalidValue;
    int nacc = 1;
    while (nacc < SB * EB) nacc *= 2;
#define LORY_SCATTER(N, B) hipLaunchKernelGGL((ms::scatter_kernel<N, B>), dim3(grid), dim3(256), lds, st, p)
    if (EB == 1) {
        switch (nacc) {
        case 1: LORY_SCATTER(1, 1); break;
        case 2: LORY_SCATTER(2, 1); break;
        case 4: LORY_SCATTER(4, 1); break;
        default: LORY_SCATTER(8, 1); break;
        }
    } else {
        switch (nacc) {
        case 2: LORY_SCATTER(2, 2); break;
        case 4: LORY_SCATTER(4, 2); break;
        default: LORY_SCATTER(8, 2); break;
        }
    }
#undef LORY_SCATTER
    return hipGetLastError();
}

hipError_t launch_dw_reduce(hipStream_t st, const float *partials, int slots, int rows, int cols,
                            float *dw, int S, int E)
{
    const int n = S * E;
    hipLaunchKernelGGL(dw_reduce_kernel, dim3((n + 255) / 256), dim3(256), 0, st, partials, slots,
                       rows, cols, dw, S, E);
    return hipGetLastError();
}

}  // namespace k
}  // namespace lory
