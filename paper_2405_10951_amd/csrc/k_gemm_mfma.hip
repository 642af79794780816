// bf16 MFMA GEMM for gfx950 (placeholder until the tiled kernels land: nothing is routed here yet).
#include "bsr_internal.h"

namespace bsr {

bool gemm_mfma_supported(const GemmDesc&) { return false; }
void gemm_mfma(const GemmDesc&, hipStream_t) {}

}  // namespace bsr
