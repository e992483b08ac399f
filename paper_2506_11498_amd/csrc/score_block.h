// Scoring of ONE lag chunk inside one workgroup of 1024 threads (Eq. 4-8 of the paper): per-channel min / max
// over the rows of the reference chunk (Eq. 4-5), the chunk's rows normalised by them (Eq. 6) and their
// standard deviation over the channels, the softmax over the chunk's tokens for K and for V, summed (Eq. 7-8).
// Used by the training-time scoring kernel (chunks of a sequence) and by the cache compression of the
// inference path (the two oldest uncompressed chunks of a cache): the same arithmetic, hence the same scores.
#pragma once
#include "common.h"

namespace lrsa {

constexpr int FUSED_THREADS = 1024;
constexpr int FUSED_MAX_L = 4096;

struct ScoreLds {
    float red[4][FUSED_THREADS / 64][128];   // per-wave partial min_K, max_K, min_V, max_V
    float s_mn[2][128], s_inv[2][128], s_den[2][128];
    float sig[2][FUSED_MAX_L];
    float sm[2 * FUSED_THREADS / 64];
};

// Kcur / Vcur: row 0 of the chunk to score, Kref / Vref: row 0 of the chunk after it; `stride` elements
// between rows; L <= FUSED_MAX_L rows each.  On return sh.sig[0][r] holds the score of row r (also written
// to out[r] when out is not null); all threads have passed a barrier after the last LDS write they depend on
// only for their own r = tid, tid + 1024, ... -- callers that read other rows synchronise first.
// sum over the 16 lanes that share a row, every lane gets the total: four rotations inside the row of 16
// (data-parallel primitive, no LDS round trip)
__device__ __forceinline__ float row16_sum(float v) {
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xf, 0xf, false));   // row_ror:8
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x124, 0xf, 0xf, false));   // row_ror:4
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x122, 0xf, 0xf, false));   // row_ror:2
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x121, 0xf, 0xf, false));   // row_ror:1
    return v;
}

// Eq. 7-8 given the standard deviations: max-subtracted softmax of sig0 over the L tokens, the same for sig1,
// their sum written to sig0[r] (and to out[r] when out is not null).  sig0, sig1: LDS, L floats each, complete
// and visible to the NT threads of the block on entry; sm: 2 * NT/64 floats of LDS.  Each thread touches only rows
// r = tid, tid + NT, ...: callers that read other rows afterwards synchronise first.
template <int NT>
__device__ __forceinline__ void softmax_sum_block(float* sig0, const float* sig1, float* sm, int L,
                                                  float* __restrict__ out) {
    constexpr int NW = NT / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // the K and the V value reduced over the block together (one pair of barriers for both)
    auto block_red2 = [&](float& a, float& b, bool is_max) {
        a = is_max ? wave_max(a) : wave_sum(a);
        b = is_max ? wave_max(b) : wave_sum(b);
        __syncthreads();
        if (lane == 0) { sm[wave] = a; sm[NW + wave] = b; }
        __syncthreads();
        float ra = sm[0], rb = sm[NW];
        for (int i = 1; i < NW; ++i) {
            ra = is_max ? fmaxf(ra, sm[i]) : ra + sm[i];
            rb = is_max ? fmaxf(rb, sm[NW + i]) : rb + sm[NW + i];
        }
        a = ra;
        b = rb;
    };
    float mk = -INFINITY, mv = -INFINITY;
    for (int r = tid; r < L; r += NT) { mk = fmaxf(mk, sig0[r]); mv = fmaxf(mv, sig1[r]); }
    block_red2(mk, mv, true);
    float zk = 0.0f, zv = 0.0f;
    for (int r = tid; r < L; r += NT) { zk += expf(sig0[r] - mk); zv += expf(sig1[r] - mv); }
    block_red2(zk, zv, false);
    for (int r = tid; r < L; r += NT) {
        const float sc = expf(sig0[r] - mk) / zk + expf(sig1[r] - mv) / zv;
        if (out) out[r] = sc;
        sig0[r] = sc;     // each thread overwrites only what it alone has read
    }
}

template <typename T>
__device__ __forceinline__ void score_chunk_block(int L, int d, int ddof, const T* __restrict__ Kcur,
                                                  const T* __restrict__ Kref, const T* __restrict__ Vcur,
                                                  const T* __restrict__ Vref, int64_t stride, ScoreLds& sh,
                                                  float* __restrict__ out) {
    constexpr int VEC = Elem<T>::VEC;
    constexpr int NW = FUSED_THREADS / 64;
    const int lpr = d / VEC;                  // lanes per row
    const int rpp = FUSED_THREADS / lpr;      // rows per pass
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = tid % lpr, rg = tid / lpr;
    const bool rows16 = lpr == 16;                  // 256-byte rows: the channel sums stay inside a row of 16 lanes
    const float inv_d = 1.0f / float(d);            // exact: head_dim is a power of two
    const float inv_dof = 1.0f / float(d - ddof);
    // ---- phase 1
    {
        float mn[2][VEC], mx[2][VEC];
#pragma unroll
        for (int z = 0; z < 2; ++z)
#pragma unroll
            for (int i = 0; i < VEC; ++i) { mn[z][i] = INFINITY; mx[z][i] = -INFINITY; }
        for (int r = rg; r < L; r += 2 * rpp) {
            // two rows of K and of V in flight
            const int r2 = r + rpp < L ? r + rpp : r;
            float k0[VEC], k1[VEC], v0[VEC], v1[VEC];
            Elem<T>::load(Kref + int64_t(r) * stride + sub * VEC, k0);
            Elem<T>::load(Vref + int64_t(r) * stride + sub * VEC, v0);
            Elem<T>::load(Kref + int64_t(r2) * stride + sub * VEC, k1);
            Elem<T>::load(Vref + int64_t(r2) * stride + sub * VEC, v1);
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                mn[0][i] = fminf(mn[0][i], fminf(k0[i], k1[i])); mx[0][i] = fmaxf(mx[0][i], fmaxf(k0[i], k1[i]));
                mn[1][i] = fminf(mn[1][i], fminf(v0[i], v1[i])); mx[1][i] = fmaxf(mx[1][i], fmaxf(v0[i], v1[i]));
            }
        }
        // lanes of one wave that hold the same channels (different rows): shuffle over the row groups
        for (int o = lpr; o < 64; o <<= 1)
#pragma unroll
            for (int z = 0; z < 2; ++z)
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    mn[z][i] = fminf(mn[z][i], __shfl_xor(mn[z][i], o, 64));
                    mx[z][i] = fmaxf(mx[z][i], __shfl_xor(mx[z][i], o, 64));
                }
        if (lane < lpr) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                sh.red[0][wave][lane * VEC + i] = mn[0][i]; sh.red[1][wave][lane * VEC + i] = mx[0][i];
                sh.red[2][wave][lane * VEC + i] = mn[1][i]; sh.red[3][wave][lane * VEC + i] = mx[1][i];
            }
        }
        __syncthreads();
        if (tid < 2 * d) {
            const int z = tid / d, c = tid % d;
            float a = INFINITY, m = -INFINITY;
            for (int w = 0; w < NW; ++w) { a = fminf(a, sh.red[2 * z][w][c]); m = fmaxf(m, sh.red[2 * z + 1][w][c]); }
            float den = m - a;
            den = den == 0.0f ? 1.0f : den;
            sh.s_mn[z][c] = a;
            sh.s_den[z][c] = den;
            sh.s_inv[z][c] = 1.0f / den;
        }
        __syncthreads();
    }
    // ---- phase 2: sigma of every row of chunk p; two rows of K and of V in flight per thread
    {
        float mn[2][VEC], den[2][VEC], inv[2][VEC];
#pragma unroll
        for (int z = 0; z < 2; ++z)
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                mn[z][i] = sh.s_mn[z][sub * VEC + i]; den[z][i] = sh.s_den[z][sub * VEC + i]; inv[z][i] = sh.s_inv[z][sub * VEC + i];
            }
        for (int r = rg; r < L; r += 2 * rpp) {
            const bool has2 = r + rpp < L;
            const int r2 = has2 ? r + rpp : r;
            float x[4][VEC];   // K row r, K row r2, V row r, V row r2
            Elem<T>::load(Kcur + int64_t(r) * stride + sub * VEC, x[0]);
            Elem<T>::load(Kcur + int64_t(r2) * stride + sub * VEC, x[1]);
            Elem<T>::load(Vcur + int64_t(r) * stride + sub * VEC, x[2]);
            Elem<T>::load(Vcur + int64_t(r2) * stride + sub * VEC, x[3]);
            float sm4[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int z = j >> 1;
                float acc = 0.0f;
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    const float a0 = x[j][i] - mn[z][i];
                    float q0 = a0 * inv[z][i];
                    q0 = __builtin_fmaf(__builtin_fmaf(-den[z][i], q0, a0), inv[z][i], q0);   // correctly rounded a0 / den
                    x[j][i] = q0;
                    acc += q0;
                }
                sm4[j] = acc;
            }
            if (rows16) {
#pragma unroll
                for (int j = 0; j < 4; ++j) sm4[j] = row16_sum(sm4[j]);
            } else {
                for (int o = lpr >> 1; o > 0; o >>= 1)
#pragma unroll
                    for (int j = 0; j < 4; ++j) sm4[j] += __shfl_xor(sm4[j], o, 64);
            }
            float var4[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float m = sm4[j] * inv_d;
                float acc = 0.0f;
#pragma unroll
                for (int i = 0; i < VEC; ++i) { const float dd = x[j][i] - m; acc += dd * dd; }
                var4[j] = acc;
            }
            if (rows16) {
#pragma unroll
                for (int j = 0; j < 4; ++j) var4[j] = row16_sum(var4[j]);
            } else {
                for (int o = lpr >> 1; o > 0; o >>= 1)
#pragma unroll
                    for (int j = 0; j < 4; ++j) var4[j] += __shfl_xor(var4[j], o, 64);
            }
            if (sub == 0) {
                sh.sig[0][r] = sqrtf(var4[0] * inv_dof);
                sh.sig[1][r] = sqrtf(var4[2] * inv_dof);
                if (has2) {
                    sh.sig[0][r2] = sqrtf(var4[1] * inv_dof);
                    sh.sig[1][r2] = sqrtf(var4[3] * inv_dof);
                }
            }
        }
        __syncthreads();
    }
    // ---- phase 3
    softmax_sum_block<FUSED_THREADS>(sh.sig[0], sh.sig[1], sh.sm, L, out);
}

}  // namespace lrsa
