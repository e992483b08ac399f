// LagKV scoring kernels (Eq. 4-8 of the paper) for gfx950.
//
// Chunks of up to 4096 tokens: ONE launch, k_score_fused, one workgroup of 1024 threads per (batch, KV head,
// chunk p): per-channel min / max over the rows of the reference chunk p+1 (Eq. 4-5), rows of chunk p
// normalised by them (Eq. 6) and their standard deviation over the channels, then the softmax over the
// chunk's tokens for K and for V, summed (Eq. 7-8); optionally the top-K selection of the chunk right away.
// Longer chunks, and shapes with so few (batch, KV head, chunk) units of at least 1024 rows that one workgroup
// each would leave more than half of the CUs idle: three launches through the workspace, the rows of a chunk cut
// into slices of 128 (256 beyond 4096 tokens),
//   k_minmax          per-channel min / max over a slice of the rows of the reference chunk p+1
//   k_sigma           rows of chunk p normalised by the combined min / max, Std over channels
//   k_softmax_select  Softmax over the L tokens of the chunk for K and for V, summed; optionally the top K
// (chunks beyond 4096 tokens: k_softmax, then the stand-alone selection kernel).
// bf16 data with head_dim 128 and chunks of 64 to 4096 rows go to the one-read kernel (score_resident.hip) instead.
// All arithmetic is fp32 on the stored values with correctly rounded division and square root, two-pass
// variance, max-subtracted softmax.  Rows are read with 16-byte loads, a row being spread over
// consecutive lanes so that a wave reads whole rows back to back.
#include "score_block.h"
#include "select_block.h"

namespace lrsa {

constexpr int SCORE_THREADS = 256;

// rows of the chunk handled by one workgroup of k_minmax / k_sigma
// (128 where the route is taken to spread few chunks over the chip, 256 for chunks beyond 4096 tokens)
__host__ __device__ inline int score_rows_per_wg(int L) { return L < 128 ? L : (L <= FUSED_MAX_L ? 128 : 256); }
__host__ __device__ inline int score_splits(int L) { int r = score_rows_per_wg(L); return (L + r - 1) / r; }

// workspace layout: mm[unit][split][2][d] floats, then sigma[unit][L] floats; unit = ((b*Hkv+h)*2+z)*Ns+p
static inline size_t mm_floats(const Dims& D) { return size_t(D.B) * D.Hkv * 2 * D.Ns * score_splits(D.L) * 2 * D.d; }
static inline size_t sigma_floats(const Dims& D) { return size_t(D.B) * D.Hkv * 2 * D.Ns * D.L; }

size_t score_ws_bytes(const Dims& D) {
    if (D.Ns == 0) return 0;
    return align256(mm_floats(D) * 4) + align256(sigma_floats(D) * 4);
}

template <typename T>
__global__ __launch_bounds__(SCORE_THREADS) void k_minmax(Dims D, const T* __restrict__ Kp, const T* __restrict__ Vp,
                                                           float* __restrict__ mm) {
    constexpr int VEC = Elem<T>::VEC;
    const int lpr = D.d / VEC;               // lanes per row
    const int rpp = SCORE_THREADS / lpr;     // rows per pass
    const int split = blockIdx.x, p = blockIdx.y;
    const int z = blockIdx.z & 1, bh = blockIdx.z >> 1;
    const int b = bh / D.Hkv, h = bh % D.Hkv;
    const T* Z = (z ? Vp : Kp) + b * D.ks[0] + h * D.ks[1];
    const int rows_wg = score_rows_per_wg(D.L);
    const int r0 = split * rows_wg;
    const int r1 = min(r0 + rows_wg, D.L);
    const int64_t base = int64_t(D.S) + int64_t(p + 1) * D.L;   // first row of the reference chunk
    const int lane = threadIdx.x % lpr, rg = threadIdx.x / lpr;

    float mn[VEC], mx[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) { mn[i] = INFINITY; mx[i] = -INFINITY; }
    for (int r = r0 + rg; r < r1; r += 4 * rpp) {       // four loads in flight; a row past the slice repeats row r
        float v[4][VEC];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            Elem<T>::load(Z + (base + (r + j * rpp < r1 ? r + j * rpp : r)) * D.ks[2] + lane * VEC, v[j]);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < VEC; ++i) { mn[i] = fminf(mn[i], v[j][i]); mx[i] = fmaxf(mx[i], v[j][i]); }
    }
    __shared__ float smn[SCORE_THREADS * 8], smx[SCORE_THREADS * 8];
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        smn[(rg * lpr + lane) * VEC + i] = mn[i];
        smx[(rg * lpr + lane) * VEC + i] = mx[i];
    }
    __syncthreads();
    if (threadIdx.x < D.d) {
        const int c = threadIdx.x;
        float a = INFINITY, bmax = -INFINITY;
        for (int g = 0; g < rpp; ++g) {
            a = fminf(a, smn[g * D.d + c]);
            bmax = fmaxf(bmax, smx[g * D.d + c]);
        }
        const int64_t unit = (int64_t(bh) * 2 + z) * D.Ns + p;
        float* out = mm + (unit * gridDim.x + split) * 2 * D.d;
        out[c] = a;
        out[D.d + c] = bmax;
    }
}

template <typename T>
__global__ __launch_bounds__(SCORE_THREADS) void k_sigma(Dims D, const T* __restrict__ Kp, const T* __restrict__ Vp,
                                                          const float* __restrict__ mm, float* __restrict__ sigma) {
    constexpr int VEC = Elem<T>::VEC;
    const int lpr = D.d / VEC;
    const int rpp = SCORE_THREADS / lpr;
    const int split = blockIdx.x, p = blockIdx.y;
    const int z = blockIdx.z & 1, bh = blockIdx.z >> 1;
    const int b = bh / D.Hkv, h = bh % D.Hkv;
    const T* Z = (z ? Vp : Kp) + b * D.ks[0] + h * D.ks[1];
    const int rows_wg = score_rows_per_wg(D.L);
    const int nsplit = gridDim.x;
    const int r0 = split * rows_wg;
    const int r1 = min(r0 + rows_wg, D.L);
    const int64_t base = int64_t(D.S) + int64_t(p) * D.L;       // first row of the scored chunk
    const int lane = threadIdx.x % lpr, rg = threadIdx.x / lpr;
    const int64_t unit = (int64_t(bh) * 2 + z) * D.Ns + p;

    // combine the partial min / max of the reference chunk: thread t reduces entry t of the 2 * d floats of a
    // partial (coalesced, the loads of different partials independent of each other), then every thread picks
    // up its own channels from LDS
    __shared__ float s_mm[2 * 128];
    if (threadIdx.x < 2 * D.d) {
        const float* src = mm + unit * nsplit * 2 * D.d + threadIdx.x;
        const bool is_min = threadIdx.x < D.d;
        float a = is_min ? INFINITY : -INFINITY;
#pragma unroll 4
        for (int s = 0; s < nsplit; ++s) {
            const float x = src[int64_t(s) * 2 * D.d];
            a = is_min ? fminf(a, x) : fmaxf(a, x);
        }
        s_mm[threadIdx.x] = a;
    }
    __syncthreads();
    float mn[VEC], den[VEC], inv[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        const int c = lane * VEC + i;
        mn[i] = s_mm[c];
        const float dd = s_mm[D.d + c] - mn[i];
        den[i] = dd == 0.0f ? 1.0f : dd;
        inv[i] = 1.0f / den[i];
    }
    const float inv_d = 1.0f / float(D.d), inv_dof = 1.0f / float(D.d - D.ddof);
    // Four rows per thread and iteration, so that four loads are in flight; a row past the slice repeats the
    // slice's last row of this thread and is not stored.  The lanes of one row run the same iterations, so
    // the shuffles stay among active lanes.  The quotient of Eq. 6 is the reciprocal product with one fused
    // residual correction, which reproduces the IEEE quotient.
    for (int r = r0 + rg; r < r1; r += 4 * rpp) {
        float v[4][VEC], s[4], q[4];
        int rr[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            rr[j] = r + j * rpp < r1 ? r + j * rpp : r;
            Elem<T>::load(Z + (base + rr[j]) * D.ks[2] + lane * VEC, v[j]);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float acc = 0.0f;
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                const float a0 = v[j][i] - mn[i];
                float q0 = a0 * inv[i];
                q0 = __builtin_fmaf(__builtin_fmaf(-den[i], q0, a0), inv[i], q0);
                v[j][i] = q0;
                acc += q0;
            }
            s[j] = acc;
        }
        for (int o = lpr >> 1; o > 0; o >>= 1)
#pragma unroll
            for (int j = 0; j < 4; ++j) s[j] += __shfl_xor(s[j], o, 64);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float mean = s[j] * inv_d;
            float acc = 0.0f;
#pragma unroll
            for (int i = 0; i < VEC; ++i) { const float dv = v[j][i] - mean; acc += dv * dv; }
            q[j] = acc;
        }
        for (int o = lpr >> 1; o > 0; o >>= 1)
#pragma unroll
            for (int j = 0; j < 4; ++j) q[j] += __shfl_xor(q[j], o, 64);
        if (lane == 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (j == 0 || r + j * rpp < r1) sigma[unit * D.L + rr[j]] = sqrtf(q[j] * inv_dof);
        }
    }
}

__device__ __forceinline__ float block_reduce(float v, bool is_max, float* sm) {
    v = is_max ? wave_max(v) : wave_sum(v);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[w] = v;
    __syncthreads();
    float r = sm[0];
    for (int i = 1; i < SCORE_THREADS / 64; ++i) r = is_max ? fmaxf(r, sm[i]) : r + sm[i];
    return r;
}

__global__ __launch_bounds__(SCORE_THREADS) void k_softmax(Dims D, const float* __restrict__ sigma,
                                                            float* __restrict__ score) {
    const int p = blockIdx.x, bh = blockIdx.y;
    const float* sk = sigma + ((int64_t(bh) * 2 + 0) * D.Ns + p) * D.L;
    const float* sv = sigma + ((int64_t(bh) * 2 + 1) * D.Ns + p) * D.L;
    __shared__ float sm[SCORE_THREADS / 64];
    float mk = -INFINITY, mv = -INFINITY;
    for (int r = threadIdx.x; r < D.L; r += SCORE_THREADS) {
        mk = fmaxf(mk, sk[r]);
        mv = fmaxf(mv, sv[r]);
    }
    mk = block_reduce(mk, true, sm);
    mv = block_reduce(mv, true, sm);
    float zk = 0.0f, zv = 0.0f;
    for (int r = threadIdx.x; r < D.L; r += SCORE_THREADS) {
        zk += expf(sk[r] - mk);
        zv += expf(sv[r] - mv);
    }
    zk = block_reduce(zk, false, sm);
    zv = block_reduce(zv, false, sm);
    float* out = score + (int64_t(bh) * D.Ns + p) * D.L;
    for (int r = threadIdx.x; r < D.L; r += SCORE_THREADS)
        out[r] = expf(sk[r] - mk) / zk + expf(sv[r] - mv) / zv;
}

// ---------------------------------------------------------------------------------------------
// Fused variant: one workgroup of 1024 threads per (batch, KV head, chunk p) does all of Eq. 4-8:
//   phase 1  per-channel min / max of K and of V over chunk p+1 (registers -> wave shuffles -> LDS)
//   phase 2  rows of chunk p normalised (Eq. 6), Std over channels -> sigma_K, sigma_V in LDS
//   phase 3  softmax over the chunk's tokens for K and V, summed, written out
// Chunk p+1 is read here as the reference and, at about the same time, by workgroup p+1 as its scored
// chunk, so the second read is served by L2 / the memory-side cache.  The division of Eq. 6 is done as
// a multiplication by the correctly rounded reciprocal plus one fused residual correction
// (q + (a - b*q) * rcp), which reproduces the IEEE quotient.
// One workgroup per (batch, KV head, chunk p).  SELECT: the workgroup also takes the top K of the chunk it has
// just scored (the scores are still in LDS).
template <typename T, bool SELECT>
__global__ __launch_bounds__(FUSED_THREADS) void k_score_fused(Dims D, const T* __restrict__ Kp,
                                                               const T* __restrict__ Vp,
                                                               float* __restrict__ score, int32_t* __restrict__ idx) {
    const int p = blockIdx.x, bh = blockIdx.y;
    const int b = bh / D.Hkv, h = bh % D.Hkv;
    const int64_t hoff = b * D.ks[0] + h * D.ks[1];
    const int64_t cur0 = int64_t(D.S) + int64_t(p) * D.L;       // first row of the scored chunk
    const int64_t ref0 = cur0 + D.L;                             // first row of the reference chunk p+1
    __shared__ ScoreLds sh;
    score_chunk_block<T>(D.L, D.d, D.ddof, Kp + hoff + cur0 * D.ks[2], Kp + hoff + ref0 * D.ks[2],
                         Vp + hoff + cur0 * D.ks[2], Vp + hoff + ref0 * D.ks[2], D.ks[2], sh,
                         score + (int64_t(bh) * D.Ns + p) * D.L);
    if (SELECT) {
        __shared__ SelectLds sel;
        __syncthreads();
        select_topk_block<FUSED_THREADS>(reinterpret_cast<const uint32_t*>(sh.sig[0]), D.L, D.K, D.S + p * D.L,
                                         idx + (int64_t(bh) * D.Ns + p) * D.K, sel);
    }
}

// Which kernels score a shape (host arithmetic; the numbers are lrsa_score_route's):
//   1  one workgroup per (batch, KV head, chunk)
//   2  sliced: one workgroup per (batch, KV head, chunk) would leave more than half of the CUs idle, and the
//      chunks are long enough (1024 rows or more) that three launches over many workgroups beat one launch over
//      few: measured at 60 units of 1024 rows, 8 + 11 + 9 us of kernel time against 43 us
//   3  one read of K and V: bf16, head_dim 128, chunks of 64 to 4096 rows; a workgroup keeps its rows in registers
//      from their min / max to their scores (score_resident.hip); taken whenever it applies
//   4  chunks beyond the LDS of the one-workgroup kernel: sliced, with softmax and selection in launches of their own
int score_route(const Dims& D) {
    if (D.Ns == 0) return 0;
    if (score_resident_applies(D)) return 3;
    if (D.L > FUSED_MAX_L) return 4;
    return int64_t(D.Ns) * D.B * D.Hkv * 2 <= 256 && D.L >= 1024 ? 2 : 1;
}

// idx != nullptr: scores AND the selection (taken by the last kernel of the route, except on route 4)
template <typename T>
static hipError_t run_score(const Dims& D, const void* K, const void* V, float* score, int32_t* idx, void* ws,
                            hipStream_t st) {
    const int route = score_route(D);
    if (route == 3) return launch_score_resident(D, K, V, score, idx, reinterpret_cast<float*>(ws), st);
    if (route == 1) {
        if (idx)
            LRSA_TIMED_LAUNCH("k_score_select_fused", st, (k_score_fused<T, true>), dim3(D.Ns, D.B * D.Hkv), dim3(FUSED_THREADS),
                              0, st, D, (const T*)K, (const T*)V, score, idx);
        else
            LRSA_TIMED_LAUNCH("k_score_fused", st, (k_score_fused<T, false>), dim3(D.Ns, D.B * D.Hkv), dim3(FUSED_THREADS), 0,
                              st, D, (const T*)K, (const T*)V, score, idx);
        return hipGetLastError();
    }
    float* mm = reinterpret_cast<float*>(ws);
    float* sigma = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + align256(mm_floats(D) * 4));
    const dim3 grid(score_splits(D.L), D.Ns, D.B * D.Hkv * 2);
    LRSA_TIMED_LAUNCH("k_minmaxT", st, k_minmax<T>, grid, dim3(SCORE_THREADS), 0, st, D, (const T*)K, (const T*)V, mm);
    LRSA_TIMED_LAUNCH("k_sigmaT", st, k_sigma<T>, grid, dim3(SCORE_THREADS), 0, st, D, (const T*)K, (const T*)V, mm, sigma);
    if (route == 2) return launch_softmax_select(D, sigma, score, idx, st);
    LRSA_TIMED_LAUNCH("k_softmax", st, k_softmax, dim3(D.Ns, D.B * D.Hkv), dim3(SCORE_THREADS), 0, st, D, sigma, score);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && idx) e = launch_select(D, score, idx, nullptr, st);
    return e;
}

hipError_t launch_score(const Dims& D, const void* K, const void* V, float* score, void* ws, hipStream_t st) {
    if (D.Ns == 0) return hipSuccess;
    return D.dtype == 1 ? run_score<bf16_t>(D, K, V, score, nullptr, ws, st) : run_score<float>(D, K, V, score, nullptr, ws, st);
}

hipError_t launch_score_select(const Dims& D, const void* K, const void* V, float* score, int32_t* idx, void* ws,
                               hipStream_t st) {
    if (D.Ns == 0) return hipSuccess;
    return D.dtype == 1 ? run_score<bf16_t>(D, K, V, score, idx, ws, st) : run_score<float>(D, K, V, score, idx, ws, st);
}

}  // namespace lrsa
