// Top-K selection per (batch, KV head, chunk) as a kernel of its own: one workgroup per lag window,
// the selection itself is select_topk_block.
#include "select_block.h"

namespace lrsa {

constexpr int SEL_THREADS = 256;

size_t select_ws_bytes(const Dims&) { return 0; }

__global__ __launch_bounds__(SEL_THREADS) void k_select(Dims D, const float* __restrict__ score,
                                                         int32_t* __restrict__ idx) {
    const int p = blockIdx.x, bh = blockIdx.y;
    const uint32_t* key = reinterpret_cast<const uint32_t*>(score) + (int64_t(bh) * D.Ns + p) * D.L;
    int32_t* out = idx + (int64_t(bh) * D.Ns + p) * D.K;
    __shared__ SelectLds sh;
    select_topk_block<SEL_THREADS>(key, D.L, D.K, D.S + p * D.L, out, sh);
}

hipError_t launch_select(const Dims& D, const float* score, int32_t* idx, void*, hipStream_t st) {
    if (D.Ns == 0) return hipSuccess;
    LRSA_TIMED_LAUNCH("k_select", st, k_select, dim3(D.Ns, D.B * D.Hkv), dim3(SEL_THREADS), 0, st, D, score, idx);
    return hipGetLastError();
}

}  // namespace lrsa
