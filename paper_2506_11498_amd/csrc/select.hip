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

// Debug aid: counts the (batch, KV head, chunk) rows of a caller-supplied idx that break the precondition of the
// attention calls -- K positions of chunk p, inside [S + pL, S + (p+1)L), strictly ascending.
__global__ void k_clear_count(int32_t* bad_rows) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *bad_rows = 0;
}
__global__ __launch_bounds__(SEL_THREADS) void k_check_idx(Dims D, const int32_t* __restrict__ idx, int32_t* bad_rows) {
    const int p = blockIdx.x, bh = blockIdx.y;
    const int32_t* row = idx + (int64_t(bh) * D.Ns + p) * D.K;
    const int lo = D.S + p * D.L, hi = lo + D.L;
    int bad = 0;
    for (int i = threadIdx.x; i < D.K; i += SEL_THREADS) {
        const int v = row[i];
        bad |= (v < lo || v >= hi) ? 1 : 0;
        if (i > 0) bad |= row[i - 1] >= v ? 1 : 0;
    }
    if (__syncthreads_or(bad) && threadIdx.x == 0) atomicAdd(bad_rows, 1);
}

hipError_t launch_check_idx(const Dims& D, const int32_t* idx, int32_t* bad_rows, hipStream_t st) {
    hipLaunchKernelGGL(k_clear_count, dim3(1), dim3(64), 0, st, bad_rows);
    if (D.Ns > 0) hipLaunchKernelGGL(k_check_idx, dim3(D.Ns, D.B * D.Hkv), dim3(SEL_THREADS), 0, st, D, idx, bad_rows);
    return hipGetLastError();
}

}  // namespace lrsa
