// Backward weight GEMM instantiations (contraction over the T tokens of a
// segment): dWg_bar = X^T dG and dWu_bar = X^T dU share X; dWd_bar = A^T dY.
#include "bf16_kernels.h"

namespace lory {
namespace k {

hipError_t launch_dwgu(hipStream_t st, const gemm::Params &p, const EpiStore2 &e)
{
    // A = X_s stored [T][d] (M contiguous), B = dG_s / dU_s stored [T][d_ff] (N contiguous)
    if (p.M % 256 == 0 && p.N % 128 == 0) return gemm::launch<256, 128, 2, 2, 1, true, true>(p, e, st);
    if (p.M % 128 == 0) return gemm::launch<128, 64, 2, 2, 1, true, true>(p, e, st);
    return gemm::launch<64, 64, 2, 2, 1, true, true>(p, e, st);
}

hipError_t launch_dwd(hipStream_t st, const gemm::Params &p, const EpiStore &e)
{
    // A = Act_s stored [T][d_ff] (M contiguous), B = dY_s stored [T][d] (N contiguous)
    if (p.N % 256 == 0 && p.M % 256 == 0) return gemm::launch<256, 256, 2, 1, 1, true, true>(p, e, st);
    if (p.N % 128 == 0) {
        if (p.M % 128 == 0) return gemm::launch<128, 128, 2, 1, 1, true, true>(p, e, st);
        return gemm::launch<64, 128, 2, 1, 1, true, true>(p, e, st);
    }
    if (p.M % 128 == 0) return gemm::launch<128, 64, 2, 1, 1, true, true>(p, e, st);
    return gemm::launch<64, 64, 2, 1, 1, true, true>(p, e, st);
}

}  // namespace k
}  // namespace lory
