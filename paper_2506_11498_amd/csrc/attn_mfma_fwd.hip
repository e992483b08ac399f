// placeholder until the MFMA kernels land
#include "common.h"
namespace lrsa {
bool mfma_supported(const Dims&) { return false; }
size_t attn_fwd_mfma_ws_bytes(const Dims&) { return 0; }
size_t attn_bwd_mfma_ws_bytes(const Dims&) { return 0; }
hipError_t launch_attn_fwd_mfma(const Dims&, const void*, const void*, const void*, const int32_t*, void*, float*, void*, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_attn_bwd_mfma(const Dims&, const void*, const void*, const void*, const void*, const void*, const float*, const int32_t*, void*, void*, void*, void*, hipStream_t) { return hipErrorNotSupported; }
}
