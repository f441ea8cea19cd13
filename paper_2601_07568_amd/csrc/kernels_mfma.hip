// bfloat16 matrix-core (MFMA) kernels for gfx950.
#include "common.h"

namespace dllm {

bool mfma_supported(const dllm_ctx* c) { return false; }

}  // namespace dllm
