// The expert-gradient kernel that keeps the per-segment weight gradients on chip
// (fused_bwd_bf16.h).
#include "bf16_kernels.h"

namespace lory {
namespace k {

bool fused_dw_fits(const fsg::Params &p) { return fsg::fits(p); }

int fused_dw_slots(const fsg::Params &p) { return fsg::grid_size(p) * 4; }

hipError_t launch_fused_dw(hipStream_t st, const fsg::Params &p)
{
    if (!fsg::fits(p)) return hipErrorInvalidValue;
    return fsg::launch(p, st);
}

}  // namespace k
}  // namespace lory
