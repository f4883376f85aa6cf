// Backward weight GEMM instantiations (contraction over the T tokens of a
// segment): dWg_bar = X^T dG and dWu_bar = X^T dU share X; dWd_bar = A^T dY.
#include "bf16_kernels.h"

namespace lory {
namespace k {

hipError_t launch_dwgu(hipStream_t st, const gemm::Params &p, const EpiStore2 &e)
{
    // A = X_s stored [T][d] (M contiguous), B = dG_s / dU_s stored [T][d_ff] (N contiguous).
    // The contraction is only T long, so the kernel is bound by writing its output: sharing X
    // between the two operand sets saves little, and two single-set launches (256-wide rows of
    // output per wave pair, half as many stores in flight per tile) measured a little faster.
    const bool split = gemm2::fits<1, 1>(p) || !gemm2::fits<2, 1>(p);
    if (!split) return gemm2::launch<2, 1, true, true>(p, e, st);
    if (gemm2::fits<1, 1>(p) || p.N % 128 == 0 || p.N % 64 != 0) {
        gemm::Params q = p;
        EpiStore e0 = {e.C0, e.c_batch, e.ldc};
        hipError_t rc = launch_dwd(st, q, e0);
        if (rc != hipSuccess) return rc;
        q.B[0] = p.B[1]; q.b_batch[0] = p.b_batch[1]; q.ldb[0] = p.ldb[1];
        EpiStore e1 = {e.C1, e.c_batch, e.ldc};
        return launch_dwd(st, q, e1);
    }
    if (p.M % 128 == 0) return gemm::launch<128, 64, 2, 2, 1, true, true>(p, e, st);
    return gemm::launch<64, 64, 2, 2, 1, true, true>(p, e, st);
}

hipError_t launch_dwd(hipStream_t st, const gemm::Params &p, const EpiStore &e)
{
    // A = Act_s stored [T][d_ff] (M contiguous), B = dY_s stored [T][d] (N contiguous)
    if (gemm2::fits<1, 1>(p)) return gemm2::launch<1, 1, true, true>(p, e, st);
    if (p.N % 128 == 0) {
        if (p.M % 128 == 0) return gemm::launch<128, 128, 2, 1, 1, true, true>(p, e, st);
        return gemm::launch<64, 128, 2, 1, 1, true, true>(p, e, st);
    }
    if (p.M % 128 == 0) return gemm::launch<128, 64, 2, 1, 1, true, true>(p, e, st);
    return gemm::launch<64, 64, 2, 1, 1, true, true>(p, e, st);
}

}  // namespace k
}  // namespace lory
