// LRSA attention forward on bf16 MFMA (gfx950), head_dim 128: Eq. 2-3 of the paper under the
// chunked mask, flash style (online softmax, only the log-sum-exp is kept for the backward).
//
// One workgroup (4 waves) owns 128 consecutive queries of one segment (the sink, or one chunk)
// of one query head; wave w owns rows 32w .. 32w+31.  The keys those queries see form one
// stream: the gather list (sink, then the survivors of the compressed chunks) followed by the
// contiguous local window up to the query itself.  Stream entry j is visible to query t iff
// j <= ng + t - cs, so only the last tiles need a mask.  The stream is walked in tiles of 64
// keys; K and V rows of a tile are fetched (gathered by position) into registers one tile
// ahead and staged row-major in LDS.
//
// Per tile and wave:  S^T = K Q^T  (keys x queries, so a lane owns one query column and the
// softmax statistics are per lane), P^T = exp2(S^T - m), O^T += V^T P^T with the accumulator
// registers of S^T reused directly as the B operand and V^T read from the row-major tile with
// transposing LDS reads.
#include "mfma_tiles.h"

namespace lrsa {

constexpr int FWD_BM = 128;   // queries per workgroup
constexpr int FWD_BN = 64;    // keys per tile
constexpr int FWD_THREADS = 256;

bool mfma_supported(const Dims& D) { return D.dtype == 1 && D.d == 128; }
size_t attn_fwd_mfma_ws_bytes(const Dims&) { return 0; }

__global__ __launch_bounds__(FWD_THREADS, 2) void k_fwd_mfma(Dims D, const bf16_t* __restrict__ Q,
                                                              const bf16_t* __restrict__ K,
                                                              const bf16_t* __restrict__ V,
                                                              const int32_t* __restrict__ idx,
                                                              bf16_t* __restrict__ O, float* __restrict__ lse,
                                                              int sink_tiles, int tpc) {
    __shared__ __attribute__((aligned(16))) unsigned char sK[FWD_BN * TILE_ROW_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char sV[FWD_BN * TILE_ROW_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int hq = blockIdx.y, b = blockIdx.z, h = hq / D.G;

    // query tile, heaviest (latest) first
    const int tix = gridDim.x - 1 - blockIdx.x;
    int qc, t0, seg_end;
    if (tix < sink_tiles) {
        qc = -1; t0 = tix * FWD_BM; seg_end = D.S < D.n ? D.S : D.n;
    } else {
        const int tt = tix - sink_tiles;
        qc = tt / tpc;
        t0 = D.S + qc * D.L + (tt % tpc) * FWD_BM;
        const int64_t e = int64_t(D.S) + int64_t(qc + 1) * D.L;
        seg_end = e < D.n ? int(e) : D.n;
    }
    if (t0 >= seg_end) return;  // uniform for the workgroup
    const int t_last = min(t0 + FWD_BM, seg_end) - 1;
    const int ng = gather_count(D, qc), cs = window_start(D, qc);
    const int m_max = ng + t_last - cs + 1;           // stream entries the last row sees
    const int ntiles = (m_max + FWD_BN - 1) / FWD_BN;

    const bf16_t* Kh = K + b * D.ks[0] + h * D.ks[1];
    const bf16_t* Vh = V + b * D.ks[0] + h * D.ks[1];
    const int32_t* idx_h = idx + (int64_t(b) * D.Hkv + h) * D.Ns * D.K;

    // this lane's query column
    const int tq = t0 + wave * 32 + l32;
    const int tq_ld = tq < t_last ? tq : t_last;
    bf16x8 qf[8];
    {
        const bf16_t* qrow = Q + b * D.qs[0] + hq * D.qs[1] + int64_t(tq_ld) * D.qs[2];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qrow + kk * 16 + g * 8);
    }
    const int lim = ng + tq - cs;                                   // last stream entry this query sees
    const int wave_first = t0 + wave * 32;
    const int wave_lim_min = ng + wave_first - cs;                  // ... the wave's first query sees
    const int wave_lim_max = ng + min(wave_first + 31, t_last) - cs;  // ... its last valid query sees

    // loader mapping: thread takes tile rows 4*kg4 .. +3, 16-byte chunk c16 of K and of V
    const int kg4 = tid >> 4, c16 = tid & 15;
    int pos0, pos1, pos2, pos3;
    uint4 kr0, kr1, kr2, kr3, vr0, vr1, vr2, vr3;
    // rows past the stream end re-read its last key; they are masked
#define LRSA_POS(tile, e) stream_pos(D, idx_h, min((tile) * FWD_BN + 4 * kg4 + (e), m_max - 1), ng, cs)
#define LRSA_FETCH_POS(tile) { pos0 = LRSA_POS(tile, 0); pos1 = LRSA_POS(tile, 1); pos2 = LRSA_POS(tile, 2); pos3 = LRSA_POS(tile, 3); }
#define LRSA_LD(base, p) (*reinterpret_cast<const uint4*>((base) + int64_t(p) * D.ks[2] + c16 * 8))
#define LRSA_ISSUE() { kr0 = LRSA_LD(Kh, pos0); kr1 = LRSA_LD(Kh, pos1); kr2 = LRSA_LD(Kh, pos2); kr3 = LRSA_LD(Kh, pos3); \
                       vr0 = LRSA_LD(Vh, pos0); vr1 = LRSA_LD(Vh, pos1); vr2 = LRSA_LD(Vh, pos2); vr3 = LRSA_LD(Vh, pos3); }
#define LRSA_ST(tile_base, e, v) (*reinterpret_cast<uint4*>((tile_base) + tile_off(4 * kg4 + (e), c16)) = (v))
#define LRSA_STASH() { LRSA_ST(sK, 0, kr0); LRSA_ST(sK, 1, kr1); LRSA_ST(sK, 2, kr2); LRSA_ST(sK, 3, kr3); \
                       LRSA_ST(sV, 0, vr0); LRSA_ST(sV, 1, vr1); LRSA_ST(sV, 2, vr2); LRSA_ST(sV, 3, vr3); }

    const float c2 = D.scale * 1.4426950408889634f;  // logits are kept in log2 units
    float m_run = -INFINITY, l_run = 0.0f;
    f32x16 o[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.0f;

    LRSA_FETCH_POS(0);
    LRSA_ISSUE();
    if (ntiles > 1) LRSA_FETCH_POS(1);
    for (int tile = 0; tile < ntiles; ++tile) {
        LRSA_STASH();
        __syncthreads();
        if (tile + 1 < ntiles) {
            LRSA_ISSUE();
            if (tile + 2 < ntiles) LRSA_FETCH_POS(tile + 2);
        }
        const int j0 = tile * FWD_BN;
        if (j0 <= wave_lim_max) {  // otherwise every key of the tile is masked for this wave
            f32x16 s[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int i = 0; i < 16; ++i) s[kb][i] = 0.0f;
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) s[kb] = mfma32(read_rows(sK, kb * 32, kk, l32, g), qf[kk], s[kb]);
            }
            float mx = -INFINITY;
            if (j0 + FWD_BN - 1 > wave_lim_min) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int j = j0 + kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
                        const float v = j <= lim ? s[kb][i] * c2 : -INFINITY;
                        s[kb][i] = v;
                        mx = fmaxf(mx, v);
                    }
            } else {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float v = s[kb][i] * c2;
                        s[kb][i] = v;
                        mx = fmaxf(mx, v);
                    }
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run, mx);   // finite: the first tile holds a visible key for every query
            const float corr = fast_exp2(m_run - m_new);
            float psum = 0.0f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float pv = fast_exp2(s[kb][i] - m_new);
                    s[kb][i] = pv;
                    psum += pv;
                }
            l_run = l_run * corr + psum;
            m_run = m_new;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[db][i] *= corr;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    const bf16x8 pf = pack8(s[kb], 8 * hh);
#pragma unroll
                    for (int db = 0; db < 4; ++db)
                        o[db] = mfma32(read_cols(sV, kb * 32 + hh * 16, db, lane), pf, o[db]);
                }
        }
        __syncthreads();
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (tq <= t_last) {
        const float inv = 1.0f / l_tot;
        bf16_t* orow = O + b * D.qs[0] + hq * D.qs[1] + int64_t(tq) * D.qs[2];
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                f32x4 v;
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = o[db][a * 4 + r] * inv;
                const bf16x4 pk = __builtin_convertvector(v, bf16x4);
                *reinterpret_cast<bf16x4*>(orow + db * 32 + a * 8 + g * 4) = pk;
            }
        if (g == 0) lse[(int64_t(b) * D.Hq + hq) * D.n + tq] = (m_run + __builtin_log2f(l_tot)) * 0.6931471805599453f;
    }
}

hipError_t launch_attn_fwd_mfma(const Dims& D, const void* Q, const void* K, const void* V, const int32_t* idx,
                                void* O, float* lse, void*, hipStream_t st) {
    const int sink_rows = D.S < D.n ? D.S : D.n;
    const int sink_tiles = (sink_rows + FWD_BM - 1) / FWD_BM;
    const int tpc = (D.L + FWD_BM - 1) / FWD_BM;
    const int tiles = sink_tiles + D.nq * tpc;
    if (tiles == 0) return hipSuccess;
    LRSA_TIMED_LAUNCH("k_fwd_mfma", st, k_fwd_mfma, dim3(tiles, D.Hq, D.B), dim3(FWD_THREADS), 0, st, D, (const bf16_t*)Q,
                       (const bf16_t*)K, (const bf16_t*)V, idx, (bf16_t*)O, lse, sink_tiles, tpc);
    return hipGetLastError();
}

}  // namespace lrsa
