// Inference-time use of LagKV compression (the setting of the paper's evaluation tables: the KV cache is
// compressed lag window by lag window while tokens are generated).
//
// Cache of one layer: Kc, Vc [B, Hkv, cap, d_h]; rows [0, len) are valid, the same len for every head:
//   sink rows | K rows per compressed chunk, chunk after chunk | uncompressed tail.
// k_cache_compress  one step for every (batch, KV head): the first L rows of the tail are scored against the
//                   next L (Eq. 4-8, the same block routine as the training-time scoring), their top K are
//                   kept in position order (text after Eq. 8) and the rest of the tail moves down by L - K
//                   rows, in place (Section 3.2, Attention Filling 1: the older chunk shrinks to its survivors,
//                   the newer one stays whole).  An optional array of original positions moves alike.
// k_decode_attn     single-query attention (Eq. 3, nothing masked) of the G query heads of a KV group over a
//                   slice of the cache rows: fp32 online softmax, partial (max, sum, output) per slice;
// k_decode_combine  merges the slices.
// Latency-shaped work: few rows, few workgroups, no matrix cores.
#include "score_block.h"
#include "select_block.h"

#include <mutex>

namespace lrsa {

constexpr int DEC_THREADS = 256;
constexpr int DEC_WAVES = DEC_THREADS / 64;
constexpr int DEC_GMAX = 8;            // query heads of a group handled per pass
constexpr int DEC_MAX_SPLITS = 256;
constexpr int DEC_U = 4;               // rows per lane group and step

static int decode_splits(const Dims& D, int len) {
    // enough workgroups to occupy the chip, at least 256 rows each
    int want = (512 + D.B * D.Hkv - 1) / (D.B * D.Hkv);
    int most = (len + 255) / 256;
    int s = want < most ? want : most;
    if (s < 1) s = 1;
    return s > DEC_MAX_SPLITS ? DEC_MAX_SPLITS : s;
}
size_t decode_ws_bytes(const Dims& D) {
    // per (batch, query head, slice): max, sum, d_h output values
    return align256(size_t(D.B) * D.Hq * DEC_MAX_SPLITS * (D.d + 2) * 4);
}
bool cache_compress_supported(const Dims& D) { return D.L <= FUSED_MAX_L && D.lp == 1; }

// ------------------------------------------------------------------------------------ compression step
// Moves rows in place: row dst0 + i <- row src(i), i = 0 .. count-1, where src(i) >= dst0 + i and src is
// increasing.  Passes of FUSED_THREADS / lpr rows, ascending; within a pass every row is read before any is
// written (a pass never writes a row that a LATER pass still has to read: its sources lie above).
template <typename T, typename SrcFn>
__device__ __forceinline__ void move_rows(T* Z, int64_t stride, int d, int dst0, int count, SrcFn src) {
    constexpr int VEC = Elem<T>::VEC;
    const int lpr = d / VEC, rpp = FUSED_THREADS / lpr;
    const int sub = threadIdx.x % lpr, rg = threadIdx.x / lpr;
    for (int i0 = 0; i0 < count; i0 += rpp) {
        const int i = i0 + rg;
        uint4 v = {0u, 0u, 0u, 0u};
        if (i < count) v = *reinterpret_cast<const uint4*>(Z + int64_t(src(i)) * stride + sub * VEC);
        __syncthreads();   // waits for the loads of every thread as well
        if (i < count) *reinterpret_cast<uint4*>(Z + int64_t(dst0 + i) * stride + sub * VEC) = v;
        __syncthreads();
    }
}
template <typename SrcFn>
__device__ __forceinline__ void move_words(int32_t* A, int dst0, int count, SrcFn src) {
    for (int i0 = 0; i0 < count; i0 += FUSED_THREADS) {
        const int i = i0 + threadIdx.x;
        int32_t v = 0;
        if (i < count) v = A[src(i)];
        __syncthreads();
        if (i < count) A[dst0 + i] = v;
        __syncthreads();
    }
}

template <typename T>
__global__ __launch_bounds__(FUSED_THREADS) void k_cache_compress(Dims D, T* __restrict__ Kc, T* __restrict__ Vc,
                                                                  int32_t* __restrict__ pos, int len, int done) {
    const int bh = blockIdx.x, b = bh / D.Hkv, h = bh % D.Hkv;
    T* Kh = Kc + b * D.ks[0] + h * D.ks[1];
    T* Vh = Vc + b * D.ks[0] + h * D.ks[1];
    const int base = D.S + D.K * done;     // first row of the chunk to compress
    __shared__ ScoreLds sh;
    __shared__ SelectLds sel;
    __shared__ int32_t keep[FUSED_MAX_L];  // the K surviving rows, relative to base, ascending
    score_chunk_block<T>(D.L, D.d, D.ddof, Kh + int64_t(base) * D.ks[2], Kh + int64_t(base + D.L) * D.ks[2],
                         Vh + int64_t(base) * D.ks[2], Vh + int64_t(base + D.L) * D.ks[2], D.ks[2], sh, nullptr);
    __syncthreads();
    select_topk_block<FUSED_THREADS>(reinterpret_cast<const uint32_t*>(sh.sig[0]), D.L, D.K, 0, keep, sel);
    __syncthreads();
    const int rest = len - (base + D.L);   // rows after the compressed chunk: they move down by L - K
    auto from_keep = [&](int i) { return base + keep[i]; };
    auto from_tail = [&](int i) { return base + D.L + i; };
    move_rows<T>(Kh, D.ks[2], D.d, base, D.K, from_keep);
    move_rows<T>(Vh, D.ks[2], D.d, base, D.K, from_keep);
    if (D.K < D.L) {
        move_rows<T>(Kh, D.ks[2], D.d, base + D.K, rest, from_tail);
        move_rows<T>(Vh, D.ks[2], D.d, base + D.K, rest, from_tail);
    }
    if (pos) {
        int32_t* ph = pos + int64_t(bh) * D.n;   // [B, Hkv, cap]
        move_words(ph, base, D.K, from_keep);
        if (D.K < D.L) move_words(ph, base + D.K, rest, from_tail);
    }
}

hipError_t launch_cache_compress(const Dims& D, void* Kc, void* Vc, int32_t* pos, int len, int done, int steps,
                                 hipStream_t st) {
    for (int s = 0; s < steps; ++s) {
        if (D.dtype == 1)
            LRSA_TIMED_LAUNCH("k_cache_compress", st, k_cache_compress<bf16_t>, dim3(D.B * D.Hkv), dim3(FUSED_THREADS), 0, st, D,
                              (bf16_t*)Kc, (bf16_t*)Vc, pos, len, done);
        else
            LRSA_TIMED_LAUNCH("k_cache_compress", st, k_cache_compress<float>, dim3(D.B * D.Hkv), dim3(FUSED_THREADS), 0, st, D,
                              (float*)Kc, (float*)Vc, pos, len, done);
        len -= D.L - D.K;
        done += 1;
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ single-query attention
// (m, l, o) of two disjoint key sets -> of their union
__device__ __forceinline__ void merge_state(float& m, float& l, float m2, float l2, float& a, float& b2) {
    const float mn = fmaxf(m, m2);
    a = m == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(m - mn);
    b2 = m2 == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(m2 - mn);
    l = l * a + l2 * b2;
    m = mn;
}

// One workgroup: the G heads of one KV group (DEC_GMAX at a time) x rows [r0, r1) of the cache.  A row is
// spread over lpr = 16-byte pieces; a wave reads 64 / lpr rows per step; logits are kept in log2 units.
template <typename T>
__global__ __launch_bounds__(DEC_THREADS) void k_decode_attn(Dims D, const T* __restrict__ q, const T* __restrict__ Kc,
                                                             const T* __restrict__ Vc, int len, int splits,
                                                             float* __restrict__ part) {
    constexpr int VEC = Elem<T>::VEC;
    const int lpr = D.d / VEC, rpw = 64 / lpr;
    const int split = blockIdx.x, bh = blockIdx.y, b = bh / D.Hkv, h = bh % D.Hkv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane % lpr, slot = lane / lpr;
    const int per = (len + splits - 1) / splits;
    const int r0 = split * per, r1 = min(len, r0 + per);
    const T* Kh = Kc + b * D.ks[0] + h * D.ks[1];
    const T* Vh = Vc + b * D.ks[0] + h * D.ks[1];
    const float c2 = D.scale * 1.4426950408889634f;
    __shared__ float sM[DEC_WAVES][DEC_GMAX], sL[DEC_WAVES][DEC_GMAX], sO[DEC_WAVES][DEC_GMAX][128];

    for (int g0 = 0; g0 < D.G; g0 += DEC_GMAX) {
        const int gn = min(DEC_GMAX, D.G - g0);
        float qv[DEC_GMAX][VEC], o[DEC_GMAX][VEC], m[DEC_GMAX], l[DEC_GMAX];
#pragma unroll
        for (int g = 0; g < DEC_GMAX; ++g) {
            m[g] = -INFINITY; l[g] = 0.0f;
#pragma unroll
            for (int i = 0; i < VEC; ++i) { o[g][i] = 0.0f; qv[g][i] = 0.0f; }
            if (g < gn) Elem<T>::load(q + (int64_t(b) * D.Hq + h * D.G + g0 + g) * D.d + sub * VEC, qv[g]);
        }
        // DEC_U rows per lane group and step: their loads are in flight together, and the running maximum is
        // refreshed (and the sums rescaled) once per step instead of once per row
        const int step = DEC_WAVES * rpw;
        for (int rb = r0 + wave * rpw + slot; rb < r1; rb += DEC_U * step) {
            float kv[DEC_U][VEC], vv[DEC_U][VEC];
#pragma unroll
            for (int u = 0; u < DEC_U; ++u) {
                const int r = min(rb + u * step, r1 - 1);   // rows past the end repeat the last one, weight 0 below
                Elem<T>::load(Kh + int64_t(r) * D.ks[2] + sub * VEC, kv[u]);
                Elem<T>::load(Vh + int64_t(r) * D.ks[2] + sub * VEC, vv[u]);
            }
#pragma unroll
            for (int g = 0; g < DEC_GMAX; ++g) {
                if (g >= gn) continue;
                float sc[DEC_U], mn = m[g];
#pragma unroll
                for (int u = 0; u < DEC_U; ++u) {
                    float t = 0.0f;
#pragma unroll
                    for (int i = 0; i < VEC; ++i) t = __builtin_fmaf(qv[g][i], kv[u][i], t);
                    sc[u] = t;
                }
                for (int off = lpr >> 1; off > 0; off >>= 1)
#pragma unroll
                    for (int u = 0; u < DEC_U; ++u) sc[u] += __shfl_xor(sc[u], off, 64);
#pragma unroll
                for (int u = 0; u < DEC_U; ++u) {
                    sc[u] = rb + u * step < r1 ? sc[u] * c2 : -INFINITY;
                    mn = fmaxf(mn, sc[u]);
                }
                const float a = __builtin_amdgcn_exp2f(m[g] - mn);   // exp2(-inf) = 0 on the first step; row rb is valid
                float ls = 0.0f;
#pragma unroll
                for (int i = 0; i < VEC; ++i) o[g][i] *= a;
#pragma unroll
                for (int u = 0; u < DEC_U; ++u) {
                    const float pr = __builtin_amdgcn_exp2f(sc[u] - mn);
                    ls += pr;
#pragma unroll
                    for (int i = 0; i < VEC; ++i) o[g][i] = __builtin_fmaf(pr, vv[u][i], o[g][i]);
                }
                l[g] = l[g] * a + ls;
                m[g] = mn;
            }
        }
        // merge the row slots of a wave, then the waves
#pragma unroll
        for (int g = 0; g < DEC_GMAX; ++g) {
            if (g >= gn) continue;
            for (int off = lpr; off < 64; off <<= 1) {
                const float m2 = __shfl_xor(m[g], off, 64), l2 = __shfl_xor(l[g], off, 64);
                float a, b2;
                merge_state(m[g], l[g], m2, l2, a, b2);
#pragma unroll
                for (int i = 0; i < VEC; ++i) o[g][i] = o[g][i] * a + __shfl_xor(o[g][i], off, 64) * b2;
            }
            if (slot == 0) {
                if (sub == 0) { sM[wave][g] = m[g]; sL[wave][g] = l[g]; }
#pragma unroll
                for (int i = 0; i < VEC; ++i) sO[wave][g][sub * VEC + i] = o[g][i];
            }
        }
        __syncthreads();
        for (int e = tid; e < gn * D.d; e += DEC_THREADS) {
            const int g = e / D.d, ch = e % D.d;
            float mm = sM[0][g], ll = sL[0][g], oo = sO[0][g][ch];
            for (int w = 1; w < DEC_WAVES; ++w) {
                float a, b2;
                merge_state(mm, ll, sM[w][g], sL[w][g], a, b2);
                oo = oo * a + sO[w][g][ch] * b2;
            }
            float* dst = part + ((int64_t(b) * D.Hq + h * D.G + g0 + g) * splits + split) * (D.d + 2);
            dst[2 + ch] = oo;
            if (ch == 0) { dst[0] = mm; dst[1] = ll; }
        }
        __syncthreads();
    }
}

template <typename T>
__global__ __launch_bounds__(128) void k_decode_combine(Dims D, const float* __restrict__ part, int splits,
                                                        T* __restrict__ O, float* __restrict__ lse) {
    const int64_t bhq = blockIdx.x;
    const int ch = threadIdx.x;
    if (ch >= D.d) return;
    const float* src = part + bhq * splits * (D.d + 2);
    float m = -INFINITY, l = 0.0f, o = 0.0f;
    for (int s = 0; s < splits; ++s) {
        float a, b2;
        merge_state(m, l, src[s * (D.d + 2)], src[s * (D.d + 2) + 1], a, b2);
        o = o * a + src[s * (D.d + 2) + 2 + ch] * b2;
    }
    Elem<T>::put(O + bhq * D.d + ch, o / l);
    if (lse && ch == 0) lse[bhq] = (m + __builtin_log2f(l)) * 0.6931471805599453f;
}

// ------------------------------------------------------------------------------------ no-allocation variant
// Scratch of lrsa_decode_attn_static: the partial (max, sum, output) records of the slices live in this array
// instead of a caller's workspace.  Every GPU holds its own copy at its own address; the array's name is only a
// host-side handle, so the device address is looked up once per device and that pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[DECODE_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};
}  // namespace

static hipError_t scratch_address(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));   // address of the current device's copy
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

size_t decode_static_need(const Dims& D, int len) {
    return size_t(D.B) * D.Hq * decode_splits(D, len) * (D.d + 2) * 4;
}

hipError_t launch_decode_attn(const Dims& D, const void* q, const void* Kc, const void* Vc, int len, void* O,
                              float* lse, void* ws, hipStream_t st);

// Same kernels, same slices, hence the same bits as launch_decode_attn; the caller has checked
// decode_static_need() <= DECODE_STATIC_SCRATCH_BYTES.  Nothing has to start at zero: every record that the
// combine kernel reads is written by the slice kernel of the same call.
hipError_t launch_decode_attn_static(const Dims& D, const void* q, const void* Kc, const void* Vc, int len, void* O,
                                     float* lse, hipStream_t st) {
    void* part = nullptr;
    const hipError_t e = scratch_address(&part);
    if (e != hipSuccess) return e;
    return launch_decode_attn(D, q, Kc, Vc, len, O, lse, part, st);
}

hipError_t launch_decode_attn(const Dims& D, const void* q, const void* Kc, const void* Vc, int len, void* O,
                              float* lse, void* ws, hipStream_t st) {
    const int splits = decode_splits(D, len);
    float* part = reinterpret_cast<float*>(ws);
    if (D.dtype == 1) {
        LRSA_TIMED_LAUNCH("k_decode_attn", st, k_decode_attn<bf16_t>, dim3(splits, D.B * D.Hkv), dim3(DEC_THREADS), 0, st, D,
                          (const bf16_t*)q, (const bf16_t*)Kc, (const bf16_t*)Vc, len, splits, part);
        LRSA_TIMED_LAUNCH("k_decode_combine", st, k_decode_combine<bf16_t>, dim3(D.B * D.Hq), dim3(128), 0, st, D, part, splits,
                          (bf16_t*)O, lse);
    } else {
        LRSA_TIMED_LAUNCH("k_decode_attn", st, k_decode_attn<float>, dim3(splits, D.B * D.Hkv), dim3(DEC_THREADS), 0, st, D,
                          (const float*)q, (const float*)Kc, (const float*)Vc, len, splits, part);
        LRSA_TIMED_LAUNCH("k_decode_combine", st, k_decode_combine<float>, dim3(D.B * D.Hq), dim3(128), 0, st, D, part, splits,
                          (float*)O, lse);
    }
    return hipGetLastError();
}

}  // namespace lrsa
