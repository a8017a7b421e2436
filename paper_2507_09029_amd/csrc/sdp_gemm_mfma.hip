// bf16 MFMA contraction for gfx950 (placeholder until the tiled kernel lands: reports every shape
// as unsupported, so the plain FMA kernel runs).
#include "sdp_internal.h"

namespace sdp {
bool gemm_mfma_supported(const GemmDesc&) { return false; }
int gemm_mfma_bf16(const GemmDesc&, hipStream_t) { return SDP_ERR_UNSUPPORTED; }
} // namespace sdp
