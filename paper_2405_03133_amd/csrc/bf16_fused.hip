// Instantiations of the merge-inside-the-GEMM kernel (fused_bf16.h): forward
// projections (expert matrices N contiguous) and the transposed uses of the
// backward (K contiguous; two sources for dX = dG Wg_bar^T + dU Wu_bar^T).
#include "bf16_kernels.h"

namespace lory {
namespace k {

namespace {
template <int NSRC, bool W_NC>
hipError_t launch_fused_t(hipStream_t st, const fmg::Params &p)
{
    // segments per task are limited by the merged tiles that fit beside the token ring in LDS
    // short segments with at most 16 experts: eight waves, two per SIMD (measured 10-25 % faster there;
    // from T = 128 on the larger tasks of the four-wave kernel win)
    if (fmg::fits8<64>(p)) return fmg::launch8<64, NSRC, W_NC>(p, st);
    if (fmg::fits<256, 1>(p)) return fmg::launch<256, 1, NSRC, W_NC>(p, st);   // T = 256
    if (fmg::fits<256, 2>(p)) return fmg::launch<256, 2, NSRC, W_NC>(p, st);   // T = 128
    if (fmg::fits<128, 1>(p)) return fmg::launch<128, 1, NSRC, W_NC>(p, st);   // T = 128, fewer tokens
    if (fmg::fits<128, 2>(p)) return fmg::launch<128, 2, NSRC, W_NC>(p, st);   // T = 64
    return hipErrorInvalidValue;
}
}  // namespace

bool fused_fits(const fmg::Params &p)
{
    return fmg::fits<256, 1>(p) || fmg::fits<256, 2>(p) || fmg::fits<128, 1>(p) || fmg::fits<128, 2>(p);
}

hipError_t launch_fused(hipStream_t st, const fmg::Params &p, int nsrc, bool w_nc)
{
    if (nsrc == 2) return w_nc ? hipErrorInvalidValue : launch_fused_t<2, false>(st, p);
    return w_nc ? launch_fused_t<1, true>(st, p) : launch_fused_t<1, false>(st, p);
}

}  // namespace k
}  // namespace lory
