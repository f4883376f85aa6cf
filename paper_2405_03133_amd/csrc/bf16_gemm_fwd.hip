// Forward GEMM instantiations: gate/up projections with the SwiGLU epilogue,
// and the down projection.
#include "bf16_kernels.h"

namespace lory {
namespace k {

namespace {
template <bool SAVE, bool ACT>
hipError_t launch_gu_t(hipStream_t st, const gemm::Params &p, const EpiGU &d)
{
    // A = X_s [T][d] (K contiguous), B = merged slabs [d][nf] (N contiguous), two sets
    const EpiGUT<SAVE, ACT> e = {d.G, d.U, d.Act, d.T, d.dff, d.n_off};
    if (gemm2::fits<2, 1>(p)) return gemm2::launch<2, 1, false, true>(p, e, st);
    if (p.M % 256 == 0 && p.N % 128 == 0) return gemm::launch<256, 128, 2, 2, 1, false, true>(p, e, st);
    if (p.M % 256 == 0) return gemm::launch<256, 64, 2, 2, 1, false, true>(p, e, st);
    if (p.M % 128 == 0) return gemm::launch<128, 64, 2, 2, 1, false, true>(p, e, st);
    return gemm::launch<64, 64, 2, 2, 1, false, true>(p, e, st);
}
}  // namespace

hipError_t launch_gu(hipStream_t st, const gemm::Params &p, const EpiGU &e)
{
    // Two output modes: G and U (the activation is then a streaming pass over them), or the
    // activation alone.  A three-plane epilogue (G, U and A at once) is not instantiated: it needs
    // scratch memory for spilled registers and measured slower than the separate pass.
    const bool save = e.G != nullptr, act = e.Act != nullptr;
    if (save == act) return hipErrorInvalidValue;
    if (act) return launch_gu_t<false, true>(st, p, e);
    return launch_gu_t<true, false>(st, p, e);
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
