// bf16 MFMA GEMM for gfx950 (placeholder until the kernel lands: reports "not supported"
// so that every caller takes the plain kernel).
#include "common.h"

namespace bf {
bool gemm_mfma_supported(int, int, int, int, int) { return false; }
bf_status gemm_mfma(int, int, const GemmArgs&, hipStream_t) { set_error("gemm_mfma: not built"); return BF_EINVAL; }
}  // namespace bf
