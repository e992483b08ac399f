// Top-K selection per (batch, KV head, chunk): the K positions of a lag window with the largest
// LagKV score (text after Eq. 8 of the paper), ties to the lowest position, written ascending.
//
// Scores are positive floats, so their bit patterns order like unsigned integers.  One workgroup
// per window finds the bit pattern of the K-th largest score with a 4-pass, 8-bit radix select
// (histogram in LDS, suffix scan over the 256 buckets), then compacts in position order: every
// score above the threshold, plus the first `need` scores equal to it.  All integer work, hence
// deterministic.
#include "common.h"

namespace lrsa {

constexpr int SEL_THREADS = 256;

size_t select_ws_bytes(const Dims&) { return 0; }

// exclusive prefix sum of `v` over the 256 threads of the block; *total receives the block sum
__device__ __forceinline__ int block_exscan(int v, int* sm /*[5]*/, int* total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int t = __shfl_up(inc, o, 64);
        if (lane >= o) inc += t;
    }
    __syncthreads();
    if (lane == 63) sm[w] = inc;
    __syncthreads();
    int off = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < SEL_THREADS / 64; ++i) {
        const int s = sm[i];
        if (i < w) off += s;
        tot += s;
    }
    *total = tot;
    return off + inc - v;
}

__global__ __launch_bounds__(SEL_THREADS) void k_select(Dims D, const float* __restrict__ score,
                                                         int32_t* __restrict__ idx) {
    const int p = blockIdx.x, bh = blockIdx.y;
    const uint32_t* key = reinterpret_cast<const uint32_t*>(score) + (int64_t(bh) * D.Ns + p) * D.L;
    int32_t* out = idx + (int64_t(bh) * D.Ns + p) * D.K;
    const int base = D.S + p * D.L;

    __shared__ int hist[256];
    __shared__ int sm[8];
    __shared__ uint32_t s_prefix;
    __shared__ int s_need;

    uint32_t prefix = 0, mask = 0;
    int need = D.K;  // how many of the elements matching `prefix` on the decided bytes are still wanted
    for (int shift = 24; shift >= 0; shift -= 8) {
        hist[threadIdx.x] = 0;
        __syncthreads();
        for (int r = threadIdx.x; r < D.L; r += SEL_THREADS) {
            const uint32_t k = key[r];
            if ((k & mask) == prefix) atomicAdd(&hist[(k >> shift) & 255], 1);
        }
        __syncthreads();
        // thread t owns bucket 255-t, so an exclusive scan counts the elements in higher buckets
        const int bucket = 255 - threadIdx.x;
        const int cnt = hist[bucket];
        int total;
        const int above = block_exscan(cnt, sm, &total);
        if (above < need && need <= above + cnt) {
            s_prefix = prefix | (uint32_t(bucket) << shift);
            s_need = need - above;
        }
        __syncthreads();
        prefix = s_prefix;
        need = s_need;
        mask |= 0xffu << shift;
        __syncthreads();
    }
    // prefix is now the K-th largest bit pattern; `need` of the elements equal to it are taken
    int written = 0, eq_seen = 0;
    for (int r0 = 0; r0 < D.L; r0 += SEL_THREADS) {
        const int r = r0 + threadIdx.x;
        const uint32_t k = r < D.L ? key[r] : 0u;
        const int is_eq = (r < D.L && k == prefix) ? 1 : 0;
        int eq_total;
        const int eq_before = block_exscan(is_eq, sm, &eq_total);
        const int take = (r < D.L && (k > prefix || (is_eq && eq_seen + eq_before < need))) ? 1 : 0;
        int take_total;
        const int pos = block_exscan(take, sm, &take_total);
        if (take) out[written + pos] = base + r;
        written += take_total;
        eq_seen += eq_total;
    }
}

hipError_t launch_select(const Dims& D, const float* score, int32_t* idx, void*, hipStream_t st) {
    if (D.Ns == 0) return hipSuccess;
    LRSA_TIMED_LAUNCH("k_select", st, k_select, dim3(D.Ns, D.B * D.Hkv), dim3(SEL_THREADS), 0, st, D, score, idx);
    return hipGetLastError();
}

}  // namespace lrsa
