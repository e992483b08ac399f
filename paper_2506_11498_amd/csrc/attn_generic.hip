// Plain fp32-arithmetic LRSA attention kernels (Eq. 2-3 of the paper under the chunked mask),
// forward and backward, for any supported dtype / head_dim.  They serve the fp32 path and are
// the fallback the MFMA kernels can be cross-checked against on the GPU.
//
// One wave works on one query row (forward, dQ) or one key column (dK, dV); its 64 lanes take
// visible keys (or visible queries) round-robin, each keeping a private online-softmax state or
// partial gradient that is combined across the wave at the end.
//
// The keys a query t in chunk q sees are enumerated as a stream: first the gather list
// "sink ++ survivors of chunks 0..q-local_prev-1" (= positions 0..S-1 followed by the flattened
// idx rows), then the contiguous window from the start of chunk q-local_prev up to t itself.
#include "common.h"

namespace lrsa {

__device__ __forceinline__ int chunk_of_pos(const Dims& D, int t) { return t < D.S ? -1 : (t - D.S) / D.L; }

// position of stream entry j for a query whose gather list has ng entries and whose window starts at cs
__device__ __forceinline__ int stream_key(const Dims& D, const int32_t* idx_h, int j, int ng, int cs) {
    if (j < ng) return j < D.S ? j : idx_h[j - D.S];
    return cs + (j - ng);
}

template <typename T, int DH>
__device__ __forceinline__ float dot_row(const float (&a)[DH], const T* __restrict__ row) {
    constexpr int VEC = Elem<T>::VEC;
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < DH; c += VEC) {
        float v[VEC];
        Elem<T>::load(row + c, v);
#pragma unroll
        for (int i = 0; i < VEC; ++i) s += a[c + i] * v[i];
    }
    return s;
}

template <typename T, int DH>
__device__ __forceinline__ void load_row(const T* __restrict__ row, float (&a)[DH]) {
    constexpr int VEC = Elem<T>::VEC;
#pragma unroll
    for (int c = 0; c < DH; c += VEC) {
        float v[VEC];
        Elem<T>::load(row + c, v);
#pragma unroll
        for (int i = 0; i < VEC; ++i) a[c + i] = v[i];
    }
}

// ------------------------------------------------------------------------------------ forward
template <typename T, int DH>
__global__ __launch_bounds__(64) void k_fwd_generic(Dims D, const T* __restrict__ Q, const T* __restrict__ K,
                                                     const T* __restrict__ V, const int32_t* __restrict__ idx,
                                                     T* __restrict__ O, float* __restrict__ lse) {
    constexpr int VEC = Elem<T>::VEC;
    const int t = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
    const int h = hq / D.G, lane = threadIdx.x;
    const T* Kh = K + b * D.ks[0] + h * D.ks[1];
    const T* Vh = V + b * D.ks[0] + h * D.ks[1];
    const int32_t* idx_h = idx + (int64_t(b) * D.Hkv + h) * D.Ns * D.K;
    const int qc = chunk_of_pos(D, t);
    const int ng = gather_count(D, qc), cs = window_start(D, qc);
    const int m = ng + (t - cs + 1);

    float q[DH];
    load_row<T, DH>(Q + b * D.qs[0] + hq * D.qs[1] + int64_t(t) * D.qs[2], q);

    float mx = -INFINITY, den = 0.0f;
    float acc[DH];
#pragma unroll
    for (int c = 0; c < DH; ++c) acc[c] = 0.0f;
    for (int j = lane; j < m; j += 64) {
        const int u = stream_key(D, idx_h, j, ng, cs);
        const float s = D.scale * dot_row<T, DH>(q, Kh + int64_t(u) * D.ks[2]);
        const float mnew = fmaxf(mx, s);
        const float corr = expf(mx - mnew), pr = expf(s - mnew);
        den = den * corr + pr;
        const T* vrow = Vh + int64_t(u) * D.ks[2];
#pragma unroll
        for (int c = 0; c < DH; c += VEC) {
            float v[VEC];
            Elem<T>::load(vrow + c, v);
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[c + i] = acc[c + i] * corr + pr * v[i];
        }
        mx = mnew;
    }
    const float M = wave_max(mx);
    const float w = expf(mx - M);  // 0 for lanes that saw no key
    const float total = wave_sum(den * w);
    float mine[DH / 64];
#pragma unroll
    for (int c = 0; c < DH; ++c) {
        const float r = wave_sum(acc[c] * w);
        if (lane == (c & 63)) mine[c >> 6] = r;
    }
    T* orow = O + b * D.qs[0] + hq * D.qs[1] + int64_t(t) * D.qs[2];
#pragma unroll
    for (int i = 0; i < DH / 64; ++i) Elem<T>::put(orow + i * 64 + lane, mine[i] / total);
    if (lane == 0) lse[(int64_t(b) * D.Hq + hq) * D.n + t] = M + logf(total);
}

// ------------------------------------------------------------------------------------ backward: dQ (and D)
template <typename T, int DH>
__global__ __launch_bounds__(64) void k_bwd_dq_generic(Dims D, const T* __restrict__ Q, const T* __restrict__ K,
                                                        const T* __restrict__ V, const T* __restrict__ O,
                                                        const T* __restrict__ dO, const float* __restrict__ lse,
                                                        const int32_t* __restrict__ idx, T* __restrict__ dQ,
                                                        float* __restrict__ Dsum) {
    constexpr int VEC = Elem<T>::VEC;
    const int t = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
    const int h = hq / D.G, lane = threadIdx.x;
    const T* Kh = K + b * D.ks[0] + h * D.ks[1];
    const T* Vh = V + b * D.ks[0] + h * D.ks[1];
    const int32_t* idx_h = idx + (int64_t(b) * D.Hkv + h) * D.Ns * D.K;
    const int qc = chunk_of_pos(D, t);
    const int ng = gather_count(D, qc), cs = window_start(D, qc);
    const int m = ng + (t - cs + 1);
    const int64_t qoff = b * D.qs[0] + hq * D.qs[1] + int64_t(t) * D.qs[2];
    const int64_t row = (int64_t(b) * D.Hq + hq) * D.n + t;

    __shared__ float sq[DH], sg[DH];
    for (int c = lane; c < DH; c += 64) {
        sq[c] = Elem<T>::get(Q + qoff + c);
        sg[c] = Elem<T>::get(dO + qoff + c);
    }
    float part = 0.0f;
    for (int c = lane; c < DH; c += 64) part += Elem<T>::get(dO + qoff + c) * Elem<T>::get(O + qoff + c);
    const float Dt = wave_sum(part);
    if (lane == 0) Dsum[row] = Dt;
    __syncthreads();
    const float l = lse[row];

    float acc[DH];
#pragma unroll
    for (int c = 0; c < DH; ++c) acc[c] = 0.0f;
    for (int j = lane; j < m; j += 64) {
        const int u = stream_key(D, idx_h, j, ng, cs);
        const T* krow = Kh + int64_t(u) * D.ks[2];
        const T* vrow = Vh + int64_t(u) * D.ks[2];
        float s = 0.0f, dp = 0.0f;
#pragma unroll
        for (int c = 0; c < DH; c += VEC) {
            float kk[VEC], vv[VEC];
            Elem<T>::load(krow + c, kk);
            Elem<T>::load(vrow + c, vv);
#pragma unroll
            for (int i = 0; i < VEC; ++i) { s += sq[c + i] * kk[i]; dp += sg[c + i] * vv[i]; }
        }
        const float pr = expf(D.scale * s - l);
        const float ds = pr * (dp - Dt);
#pragma unroll
        for (int c = 0; c < DH; c += VEC) {
            float kk[VEC];
            Elem<T>::load(krow + c, kk);
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[c + i] += ds * kk[i];
        }
    }
    float mine[DH / 64];
#pragma unroll
    for (int c = 0; c < DH; ++c) {
        const float r = wave_sum(acc[c]);
        if (lane == (c & 63)) mine[c >> 6] = r;
    }
#pragma unroll
    for (int i = 0; i < DH / 64; ++i) Elem<T>::put(dQ + qoff + i * 64 + lane, D.scale * mine[i]);
}

// ------------------------------------------------------------------------------------ backward: dK, dV
// is position u (in a scored chunk) one of the survivors?  idx rows are ascending: binary search
__device__ __forceinline__ bool is_survivor(const Dims& D, const int32_t* idx_h, int u) {
    const int c = (u - D.S) / D.L;
    if (c >= D.Ns) return false;
    const int32_t* rowp = idx_h + int64_t(c) * D.K;
    int lo = 0, hi = D.K - 1;
    while (lo <= hi) {
        const int mid = (lo + hi) >> 1;
        const int v = rowp[mid];
        if (v == u) return true;
        if (v < u) lo = mid + 1; else hi = mid - 1;
    }
    return false;
}

template <typename T, int DH>
__global__ __launch_bounds__(64) void k_bwd_dkv_generic(Dims D, const T* __restrict__ Q, const T* __restrict__ K,
                                                         const T* __restrict__ V, const T* __restrict__ dO,
                                                         const float* __restrict__ lse, const float* __restrict__ Dsum,
                                                         const int32_t* __restrict__ idx, T* __restrict__ dK,
                                                         T* __restrict__ dV) {
    constexpr int VEC = Elem<T>::VEC;
    const int u = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x;
    const int32_t* idx_h = idx + (int64_t(b) * D.Hkv + h) * D.Ns * D.K;
    const int64_t koff = b * D.ks[0] + h * D.ks[1] + int64_t(u) * D.ks[2];

    __shared__ float sk[DH], sv[DH];
    for (int c = lane; c < DH; c += 64) {
        sk[c] = Elem<T>::get(K + koff + c);
        sv[c] = Elem<T>::get(V + koff + c);
    }
    __syncthreads();
    // rows that see u: all later rows for sink tokens and survivors, else up to the end of the
    // last chunk that still holds u's chunk in full
    int end = D.n;
    if (u >= D.S && !is_survivor(D, idx_h, u)) {
        const int64_t e = int64_t(D.S) + (int64_t((u - D.S) / D.L) + 1 + D.lp) * D.L;
        end = e < D.n ? int(e) : D.n;
    }
    const int len = end - u;
    const int64_t total = int64_t(len) * D.G;

    float dk[DH], dv[DH];
#pragma unroll
    for (int c = 0; c < DH; ++c) { dk[c] = 0.0f; dv[c] = 0.0f; }
    for (int64_t j = lane; j < total; j += 64) {
        const int g = int(j / len), t = u + int(j % len);
        const int hq = h * D.G + g;
        const int64_t qoff = b * D.qs[0] + hq * D.qs[1] + int64_t(t) * D.qs[2];
        const int64_t row = (int64_t(b) * D.Hq + hq) * D.n + t;
        const T* qrow = Q + qoff;
        const T* grow = dO + qoff;
        float s = 0.0f, dp = 0.0f;
#pragma unroll
        for (int c = 0; c < DH; c += VEC) {
            float qq[VEC], gg[VEC];
            Elem<T>::load(qrow + c, qq);
            Elem<T>::load(grow + c, gg);
#pragma unroll
            for (int i = 0; i < VEC; ++i) { s += qq[i] * sk[c + i]; dp += gg[i] * sv[c + i]; }
        }
        const float pr = expf(D.scale * s - lse[row]);
        const float ds = pr * (dp - Dsum[row]);
#pragma unroll
        for (int c = 0; c < DH; c += VEC) {
            float qq[VEC], gg[VEC];
            Elem<T>::load(qrow + c, qq);
            Elem<T>::load(grow + c, gg);
#pragma unroll
            for (int i = 0; i < VEC; ++i) { dk[c + i] += ds * qq[i]; dv[c + i] += pr * gg[i]; }
        }
    }
    float mk[DH / 64], mv[DH / 64];
#pragma unroll
    for (int c = 0; c < DH; ++c) {
        const float a = wave_sum(dk[c]);
        const float e = wave_sum(dv[c]);
        if (lane == (c & 63)) { mk[c >> 6] = a; mv[c >> 6] = e; }
    }
#pragma unroll
    for (int i = 0; i < DH / 64; ++i) {
        Elem<T>::put(dK + koff + i * 64 + lane, D.scale * mk[i]);
        Elem<T>::put(dV + koff + i * 64 + lane, mv[i]);
    }
}

// ------------------------------------------------------------------------------------ launchers
size_t attn_fwd_generic_ws_bytes(const Dims&) { return 0; }
size_t attn_bwd_generic_ws_bytes(const Dims& D) { return align256(size_t(D.B) * D.Hq * D.n * 4); }

template <typename T, int DH>
static hipError_t run_fwd(const Dims& D, const void* Q, const void* K, const void* V, const int32_t* idx, void* O,
                          float* lse, hipStream_t st) {
    LRSA_TIMED_LAUNCH("k_fwd_genericT", st, (k_fwd_generic<T, DH>), dim3(D.n, D.Hq, D.B), dim3(64), 0, st, D, (const T*)Q, (const T*)K,
                       (const T*)V, idx, (T*)O, lse);
    return hipGetLastError();
}

template <typename T, int DH>
static hipError_t run_bwd(const Dims& D, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                          const float* lse, const int32_t* idx, void* dQ, void* dK, void* dV, void* ws,
                          hipStream_t st) {
    float* Dsum = reinterpret_cast<float*>(ws);
    LRSA_TIMED_LAUNCH("k_bwd_dq_genericT", st, (k_bwd_dq_generic<T, DH>), dim3(D.n, D.Hq, D.B), dim3(64), 0, st, D, (const T*)Q, (const T*)K,
                       (const T*)V, (const T*)O, (const T*)dO, lse, idx, (T*)dQ, Dsum);
    LRSA_TIMED_LAUNCH("k_bwd_dkv_genericT", st, (k_bwd_dkv_generic<T, DH>), dim3(D.n, D.Hkv, D.B), dim3(64), 0, st, D, (const T*)Q,
                       (const T*)K, (const T*)V, (const T*)dO, lse, Dsum, idx, (T*)dK, (T*)dV);
    return hipGetLastError();
}

hipError_t launch_attn_fwd_generic(const Dims& D, const void* Q, const void* K, const void* V, const int32_t* idx,
                                   void* O, float* lse, void*, hipStream_t st) {
    if (D.dtype == 0) return D.d == 64 ? run_fwd<float, 64>(D, Q, K, V, idx, O, lse, st)
                                       : run_fwd<float, 128>(D, Q, K, V, idx, O, lse, st);
    return D.d == 64 ? run_fwd<bf16_t, 64>(D, Q, K, V, idx, O, lse, st)
                     : run_fwd<bf16_t, 128>(D, Q, K, V, idx, O, lse, st);
}

hipError_t launch_attn_bwd_generic(const Dims& D, const void* Q, const void* K, const void* V, const void* O,
                                   const void* dO, const float* lse, const int32_t* idx, void* dQ, void* dK,
                                   void* dV, void* ws, hipStream_t st) {
    if (D.dtype == 0)
        return D.d == 64 ? run_bwd<float, 64>(D, Q, K, V, O, dO, lse, idx, dQ, dK, dV, ws, st)
                         : run_bwd<float, 128>(D, Q, K, V, O, dO, lse, idx, dQ, dK, dV, ws, st);
    return D.d == 64 ? run_bwd<bf16_t, 64>(D, Q, K, V, O, dO, lse, idx, dQ, dK, dV, ws, st)
                     : run_bwd<bf16_t, 128>(D, Q, K, V, O, dO, lse, idx, dQ, dK, dV, ws, st);
}

}  // namespace lrsa
