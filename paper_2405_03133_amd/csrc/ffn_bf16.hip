// placeholder, replaced below
#include "lory_internal.h"
namespace lory {
size_t bf16_workspace_bytes(const Dims &, int) { return 256; }
int bf16_ffn_fwd(const Dims &, const void *, const float *, const void *, const void *, const void *, void *, void *, void *, void *, hipStream_t) { return LORY_ERR_DTYPE; }
int bf16_ffn_bwd(const Dims &, const void *, const float *, const void *, const void *, const void *, const void *, const void *, const void *, void *, void *, void *, void *, int, int, float *, void *, hipStream_t) { return LORY_ERR_DTYPE; }
}
