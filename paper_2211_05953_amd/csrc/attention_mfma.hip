// bf16 MFMA attention for gfx950 (placeholder until the kernel lands).
#include "common.h"

namespace bf {
bool attention_mfma_supported(int, int) { return false; }
bf_status attention_fwd_mfma(int, int, int, int, int, const void*, void*, float*, hipStream_t) { set_error("attention_mfma: not built"); return BF_EINVAL; }
bf_status attention_bwd_mfma(int, int, int, int, int, const void*, const void*, const float*, const void*, void*, float*, hipStream_t) { set_error("attention_mfma: not built"); return BF_EINVAL; }
}  // namespace bf
