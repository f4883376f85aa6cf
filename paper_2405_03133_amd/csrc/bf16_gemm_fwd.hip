// Forward GEMM instantiations: gate/up projections with the SwiGLU epilogue,
// and the down projection.
#include "bf16_kernels.h"

namespace lory {
namespace k {

hipError_t launch_gu(hipStream_t st, const gemm::Params &p, const EpiGU &e)
{
    // A = X_s [T][d] (K contiguous), B = merged slabs [d][nf] (N contiguous), two sets
    if (gemm2::fits<2, 1>(p)) return gemm2::launch<2, 1, false, true>(p, e, st);
    if (p.M % 256 == 0 && p.N % 128 == 0) return gemm::launch<256, 128, 2, 2, 1, false, true>(p, e, st);
    if (p.M % 256 == 0) return gemm::launch<256, 64, 2, 2, 1, false, true>(p, e, st);
    if (p.M % 128 == 0) return gemm::launch<128, 64, 2, 2, 1, false, true>(p, e, st);
    return gemm::launch<64, 64, 2, 2, 1, false, true>(p, e, st);
}

hipError_t launch_down(hipStream_t st, const gemm::Params &p, const EpiStore &e)
{
    // A = Act_s [T][d_ff], B = merged slab [d_ff][jf] (N contiguous)
    if (gemm2::fits<1, 1>(p)) return gemm2::launch<1, 1, false, true>(p, e, st);
    if (p.N % 256 == 0 && p.M % 256 == 0) return gemm::launch<256, 256, 2, 1, 1, false, true>(p, e, st);
    if (p.N % 128 == 0) {
        if (p.M % 256 == 0) return gemm::launch<256, 128, 2, 1, 1, false, true>(p, e, st);
        if (p.M % 128 == 0) return gemm::launch<128, 128, 2, 1, 1, false, true>(p, e, st);
        return gemm::launch<64, 128, 2, 1, 1, false, true>(p, e, st);
    }
    if (p.M % 256 == 0) return gemm::launch<256, 64, 2, 1, 1, false, true>(p, e, st);
    if (p.M % 128 == 0) return gemm::launch<128, 64, 2, 1, 1, false, true>(p, e, st);
    return gemm::launch<64, 64, 2, 1, 1, false, true>(p, e, st);
}

}  // namespace k
}  // namespace lory
