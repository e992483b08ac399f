// Top-K of one lag window inside one workgroup (text after Eq. 8 of the paper): the K positions with the
// largest score, ties to the lowest position, written ascending.
//
// Scores are positive floats, so their bit patterns order like unsigned integers.  The workgroup finds
// the bit pattern of the K-th largest score with an 8-bit radix select (histogram in LDS, suffix scan over
// the 256 buckets), then compacts in position order: every score above the threshold, plus the first
// `need` scores equal to it.  The scores of one chunk share their sign and most of their exponent, so the
// digits are taken from (pattern - smallest pattern of the chunk), shifted left until the span's top bit is
// bit 31: the first histogram then spreads over the buckets instead of piling its LDS atomics on one or two
// addresses, and a narrow span needs fewer than four passes.  The map is monotone and one-to-one, so the
// order, the ties and hence the selection are unchanged.  The passes stop as soon as the bucket that holds the
// K-th largest element is wanted whole (after two bytes it usually holds that element alone): the bytes below
// would only order elements that are all taken.  All integer work, hence deterministic.  Used by the
// stand-alone selection kernel (keys in global memory) and by the scoring kernels (keys in LDS).
#pragma once
#include "common.h"

namespace lrsa {

struct SelectLds {
    int hist[256];
    int sm[16];
    uint32_t prefix;
    int need;
    int all;      // every element of the chosen bucket is wanted: the lower bytes decide nothing
};

// exclusive prefix sum of `v` over the NT threads of the block; *total receives the block sum
template <int NT>
__device__ __forceinline__ int block_exscan(int v, int* sm /*[NT/64]*/, int* total) {
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
    for (int i = 0; i < NT / 64; ++i) {
        const int s = sm[i];
        if (i < w) off += s;
        tot += s;
    }
    *total = tot;
    return off + inc - v;
}

// key: L bit patterns (global or LDS); out: K positions base + r, ascending.  Every thread of the block calls.
template <int NT>
__device__ __forceinline__ void select_topk_block(const uint32_t* key, int L, int K, int base, int32_t* out,
                                                  SelectLds& sh) {
    static_assert(NT >= 256 && NT % 64 == 0 && NT <= 1024, "block size");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int NW = NT / 64;
    // smallest and largest pattern of the chunk
    uint32_t lo = 0xffffffffu, hi = 0u;
    for (int r = tid; r < L; r += NT) {
        const uint32_t k = key[r];
        lo = k < lo ? k : lo;
        hi = k > hi ? k : hi;
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t a = uint32_t(__shfl_xor(int(lo), o, 64)), b = uint32_t(__shfl_xor(int(hi), o, 64));
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }
    if (lane == 0) { sh.hist[wave] = int(lo); sh.hist[NW + wave] = int(hi); }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        const uint32_t a = uint32_t(sh.hist[i]), b = uint32_t(sh.hist[NW + i]);
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }
    __syncthreads();      // the histogram is cleared next
    const uint32_t span = hi - lo;
    const int lsh = span ? __builtin_clz(span) : 31;            // (k - lo) << lsh puts the span's top bit at bit 31
    const int low_zero = lsh >> 3;                              // low bytes that are zero for every key: no pass
    auto rel = [&](uint32_t k) { return (k - lo) << lsh; };
    uint32_t prefix = 0, mask = 0;
    int need = K;  // how many of the elements matching `prefix` on the decided bytes are still wanted
    for (int shift = 24; shift >= 8 * low_zero; shift -= 8) {
        if (tid < 256) sh.hist[tid] = 0;
        __syncthreads();
        for (int r = tid; r < L; r += NT) {
            const uint32_t k = rel(key[r]);
            if ((k & mask) == prefix) atomicAdd(&sh.hist[(k >> shift) & 255], 1);
        }
        __syncthreads();
        // the first wave walks the buckets from the top: lane l owns buckets 255-4l .. 252-4l, an exclusive
        // scan over the lanes counts the elements in higher buckets
        if (tid < 64) {
            int c[4], tot = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) { c[i] = sh.hist[255 - 4 * lane - i]; tot += c[i]; }
            int inc = tot;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(inc, o, 64);
                if (lane >= o) inc += t;
            }
            int above = inc - tot;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (above < need && need <= above + c[i]) {
                    sh.prefix = prefix | (uint32_t(255 - 4 * lane - i) << shift);
                    sh.need = need - above;
                    sh.all = need - above == c[i] ? 1 : 0;
                }
                above += c[i];
            }
        }
        __syncthreads();
        prefix = sh.prefix;
        need = sh.need;
        mask |= 0xffu << shift;
        if (sh.all) break;
    }
    // On the decided bytes (`mask`), `prefix` is the pattern of the K-th largest element; `need` of the elements
    // that equal it there are taken, the first ones in position order (all of them after an early stop).  Every
    // thread takes SEL_RUN consecutive positions, so that one packed scan serves SEL_RUN * NT elements: larger
    // ones in the low half-word, equal ones in the high half-word.
    constexpr int SEL_RUN = 4;
    int gt_seen = 0, eq_seen = 0;
    for (int b0 = 0; b0 < L; b0 += SEL_RUN * NT) {
        const int r0 = b0 + tid * SEL_RUN;
        uint32_t km[SEL_RUN];
        int ngt = 0, neq = 0;
#pragma unroll
        for (int i = 0; i < SEL_RUN; ++i) {
            km[i] = r0 + i < L ? rel(key[r0 + i]) & mask : 0u;
            ngt += (r0 + i < L && km[i] > prefix) ? 1 : 0;
            neq += (r0 + i < L && km[i] == prefix) ? 1 : 0;
        }
        int total;
        const int before = block_exscan<NT>(ngt | (neq << 16), sh.sm, &total);
        int g = gt_seen + (before & 0xffff), e = eq_seen + (before >> 16);
#pragma unroll
        for (int i = 0; i < SEL_RUN; ++i) {
            if (r0 + i >= L) break;
            const bool is_gt = km[i] > prefix, is_eq = km[i] == prefix;
            if (is_gt || (is_eq && e < need)) out[g + min(e, need)] = base + r0 + i;
            g += is_gt ? 1 : 0;
            e += is_eq ? 1 : 0;
        }
        gt_seen += total & 0xffff;
        eq_seen += total >> 16;
    }
}

}  // namespace lrsa
