// Backward data GEMM instantiations: dA = dY Wd_bar^T and dX = dG Wg_bar^T + dU Wu_bar^T.
#include "bf16_kernels.h"

namespace lory {
namespace k {

hipError_t launch_da(hipStream_t st, const gemm::Params &p, const EpiStore &e)
{
    // A = dY_s [T][d], B = merged slab rows [nf][d] (K contiguous)
    if (gemm2::fits<1, 1>(p)) return gemm2::launch<1, 1, false, false>(p, e, st);
    if (p.N % 128 == 0) {
        if (p.M % 256 == 0) return gemm::launch<256, 128, 2, 1, 1, false, false>(p, e, st);
        if (p.M % 128 == 0) return gemm::launch<128, 128, 2, 1, 1, false, false>(p, e, st);
        return gemm::launch<64, 128, 2, 1, 1, false, false>(p, e, st);
    }
    if (p.M % 256 == 0) return gemm::launch<256, 64, 2, 1, 1, false, false>(p, e, st);
    if (p.M % 128 == 0) return gemm::launch<128, 64, 2, 1, 1, false, false>(p, e, st);
    return gemm::launch<64, 64, 2, 1, 1, false, false>(p, e, st);
}

hipError_t launch_dx(hipStream_t st, const gemm::Params &p, const EpiStore &e)
{
    // two sources: (dG_s, Wg_bar rows [kf][d_ff]) and (dU_s, Wu_bar rows), all K contiguous
    if (gemm2::fits<1, 2>(p)) return gemm2::launch<1, 2, false, false>(p, e, st);
    if (p.N % 256 == 0 && p.M % 256 == 0) return gemm::launch<256, 256, 2, 1, 2, false, false>(p, e, st);
    if (p.N % 128 == 0) {
        if (p.M % 256 == 0) return gemm::launch<256, 128, 2, 1, 2, false, false>(p, e, st);
        if (p.M % 128 == 0) return gemm::launch<128, 128, 2, 1, 2, false, false>(p, e, st);
        return gemm::launch<64, 128, 2, 1, 2, false, false>(p, e, st);
    }
    if (p.M % 256 == 0) return gemm::launch<256, 64, 2, 1, 2, false, false>(p, e, st);
    if (p.M % 128 == 0) return gemm::launch<128, 64, 2, 1, 2, false, false>(p, e, st);
    return gemm::launch<64, 64, 2, 1, 2, false, false>(p, e, st);
}

}  // namespace k
}  // namespace lory
