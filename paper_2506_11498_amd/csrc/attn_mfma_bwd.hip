// LRSA attention backward on bf16 MFMA (gfx950), head_dim 128.  Gradients of sum(O * dO) with
// the mask constant:  A = exp(scale Q K^T + M - lse), dV = A^T dO, dA = dO V^T,
// D = rowsum(dO * O), dS = A * (dA - D), dQ = scale dS K, dK = scale dS^T Q.
//
// Deterministic, no atomics.  Three launches on one stream:
//   k_bwd_dq          query-outer: a workgroup owns 256 (head, query) rows of one KV group and walks their
//                     key stream exactly like the forward (gather list, then the local window), recomputing A;
//                     it also leaves D[b,hq,t] = dO[t] . O[t] and lse in log2 units in the workspace
//   k_bwd_dkv         key-outer, two kinds of workgroups in one launch.  GATHER: 256 consecutive entries of one
//                     KV head's gather list (sink ++ survivors) x one slice of query chunks -> fp32 partial
//                     dK, dV rows in the workspace.  WINDOW: 256 consecutive positions x the queries that see
//                     them through the local window (own chunk causally, the next local_prev chunks in full);
//                     positions outside the gather list are written as final dK, dV, listed ones as one more
//                     fp32 partial.
//   k_bwd_dkv_reduce  listed positions: window partial + the slices, in a fixed order -> dK, dV
// In the key-outer kernel a lane owns one key column of S = Q K^T: K fragments stay in registers for the
// whole walk, the workgroup's V rows in LDS; Q and dO rows stream through LDS 64 rows at a time and are read
// both row-wise (for S and dA) and transposed (for dV^T += dO^T A and dK^T += Q^T dS).
#include "mfma_tiles.h"

namespace lrsa {

constexpr int KV_WAVES = 8;              // waves per workgroup of the key-outer kernel (two per SIMD)
constexpr int KV_THREADS = 64 * KV_WAVES;
constexpr int DQ_BN = 64;
constexpr int DQ_PF = 4;                 // LDS operands of the query-outer kernel are read this many MFMAs ahead
constexpr int DQ_WAVES = 8;              // waves per workgroup of the query-outer kernel (two per SIMD)
constexpr int DQ_THREADS = 64 * DQ_WAVES;
constexpr int KV_NB = 1;                        // 32-key blocks per wave (2 needs one wave per SIMD: measured slower)
constexpr int KV_BK = 32 * KV_NB * KV_WAVES;   // keys per workgroup
constexpr int KV_BQ = 32;   // query rows per MFMA sub-step
constexpr int KV_SUB = 2;   // sub-steps per pipeline step (one LDS stage, one barrier)
constexpr int KV_ROWS = KV_BQ * KV_SUB;   // query rows per step
constexpr int KV_MAX_SLICES = 16;

// ------------------------------------------------------------------------------------ host-side plan
struct BwdPlan {
    int sink_tiles_k, tpc_k;    // dK/dV window mode: key tiles of KV_BK positions in the sink / per chunk
    int kc_lo, ktiles;          // first key chunk and number of key tiles of the window part
    int fq0, fq1;               // query chunks whose rows take part (all of them unless a row window is set)
    int gl_total, gtiles;       // gather list length per KV head as the last query chunk sees it, its tiles
    int qch, nsl;               // query chunks per slice, slices per gather tile (<= KV_MAX_SLICES)
    int gather_wgs;             // workgroups of the GATHER part of the dK/dV launch (a multiple of 8)
    size_t off_lse2, off_part, off_compact, off_dkc, bytes;   // workspace: D, lse in log2 units, the fp32 partials,
                                                              // condensed K/V, condensed dK/dV (fp32)
};

static BwdPlan make_plan(const Dims& D) {
    BwdPlan P;
    const int sink_rows = D.S < D.n ? D.S : D.n;
    P.fq0 = D.fq0;
    P.fq1 = D.fq1;
    const int nqf = D.fq1 - D.fq0;                 // query chunks in the window
    P.sink_tiles_k = D.row_begin == 0 ? (sink_rows + KV_BK - 1) / KV_BK : 0;   // sink keys see only sink queries here
    P.tpc_k = (D.L + KV_BK - 1) / KV_BK;
    P.kc_lo = D.fq0 - D.lp > 0 ? D.fq0 - D.lp : 0;  // the local window reaches lp chunks back
    P.ktiles = P.sink_tiles_k + (D.fq1 - P.kc_lo) * P.tpc_k;
    P.gl_total = D.fq1 > 0 ? gather_count(D, D.fq1 - 1) : 0;
    P.gtiles = (P.gl_total + KV_BK - 1) / KV_BK;
    // aim at ~8192 query rows (x G heads) per workgroup, but never more than KV_MAX_SLICES slices
    int64_t qch = (256 * 32) / (int64_t(D.L) * D.G);
    if (qch < 1) qch = 1;
    const int min_qch = (nqf + KV_MAX_SLICES - 1) / KV_MAX_SLICES;
    if (qch < min_qch) qch = min_qch;
    if (qch < 1) qch = 1;
    // small problems: shorter slices (down to ~1024 query rows x G heads) until the gather workgroups -- about
    // half of the (tile, slice) grid sees any query -- fill the chip twice
    while (qch > min_qch && qch > 1 && (qch / 2) * int64_t(D.L) * D.G >= 1024 &&
           int64_t(D.B) * D.Hkv * P.gtiles * ((nqf + qch - 1) / qch) / 2 < 512)
        qch /= 2;
    P.qch = int(qch);
    P.nsl = nqf > 0 ? (nqf + P.qch - 1) / P.qch : 0;
    P.off_lse2 = align256(size_t(D.B) * D.Hq * D.lse_stride * 4);
    P.off_part = 2 * P.off_lse2;
    P.gather_wgs = P.gtiles > 0 ? (D.B * D.Hkv * P.nsl + 7) / 8 * 8 * P.gtiles : 0;
    // slots 0 .. nsl-1: the GATHER workgroups' slices; slot nsl: what the WINDOW workgroups add to listed positions
    const size_t part = size_t(2) * (P.nsl + 1) * D.B * D.Hkv * P.gl_total * 128 * 4;
    P.off_compact = P.off_part + align256(part);
    P.off_dkc = P.off_compact + compact_kv_bytes(D);
    P.bytes = P.off_dkc + (D.compact ? 2 * align256(size_t(D.B) * D.Hkv * P.gl_total * 128 * 4) : 0);
    return P;
}

size_t attn_bwd_mfma_ws_bytes(const Dims& D) { return make_plan(D).bytes; }

// ------------------------------------------------------------------------------------ dQ
// One 64-key tile for one wave: per 32 keys S^T and dA^T, then dS^T, then dQ^T += K^T dS^T.
// MASK: the tile holds entries some query of the wave does not see (only the last tiles of a walk).
template <bool MASK>
__device__ __forceinline__ void dq_tile(const unsigned char* sK, const unsigned char* sV, const bf16x8 (&qf)[8],
                                        const bf16x8 (&gf)[8], const LaneOffs& lo, f32x16 (&dq)[4], int j0, int lim,
                                        int wave_lim_max, float c2, float lse2, float Dq, int lane) {
    const int g = lane >> 5;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        if (!MASK || j0 + kb * 32 <= wave_lim_max) {  // otherwise these 32 keys are masked for the whole wave
            // 24 MFMAs: S^T (K rows), dA^T (V rows), dQ^T (K transposed, rows 0-15 then 16-31); their LDS operands
            // form one stream that is read DQ_PF ahead.  A = exp2(S*c2 - lse2) is written beside the dA MFMAs it
            // does not depend on.
            f32x16 s, dp;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s[i] = 0.0f; dp[i] = 0.0f; }
#define LRSA_DQ_OPND(n)                                                                                      \
    ((n) < 8 ? read_rows_o(sK, lo, kb * 32, (n)) : (n) < 16 ? read_rows_o(sV, lo, kb * 32, (n) - 8)           \
             : read_cols_o(sK, lo, kb * 32 + ((n) >= 20 ? 16 : 0), (n) & 3))
            bf16x8 a[DQ_PF];
#pragma unroll
            for (int n = 0; n < DQ_PF; ++n) a[n] = LRSA_DQ_OPND(n);
            const float neg_l = -lse2;
            bf16x8 dsf0, dsf1;
#pragma unroll
            for (int n = 0; n < 24; ++n) {
                if (n < 8) s = mfma32(a[n % DQ_PF], qf[n], s);
                else if (n < 16) dp = mfma32(a[n % DQ_PF], gf[n - 8], dp);
                else if (n < 20) dq[n - 16] = mfma32(a[n % DQ_PF], dsf0, dq[n - 16]);
                else dq[n - 20] = mfma32(a[n % DQ_PF], dsf1, dq[n - 20]);
                if (n + DQ_PF < 24) a[n % DQ_PF] = LRSA_DQ_OPND(n + DQ_PF);
                if (n >= 8 && n < 16) {
#pragma unroll
                    for (int i = 2 * (n - 8); i < 2 * (n - 8) + 2; ++i) {
                        float pr = fast_exp2(__builtin_fmaf(s[i], c2, neg_l));
                        if (MASK) {
                            const int j = j0 + kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
                            pr = j <= lim ? pr : 0.0f;
                        }
                        s[i] = pr;
                    }
                }
                if (n == 15) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) s[i] *= dp[i] - Dq;
                    dsf0 = pack8(s, 0);
                    dsf1 = pack8(s, 8);
                }
            }
#undef LRSA_DQ_OPND
        }
    }
}

// A tile all of whose 64 keys every query of the wave sees: both 32-key halves as ONE stream of 48 MFMAs,
//   S0 | dA0 (+ exp of half 0) | S1 (+ dS of half 0) | dA1 (+ exp of half 1) | dQ0 (+ dS of half 1) | dQ1,
// so that every piece of vector work sits beside MFMAs it does not depend on.  LDS operands are read DQ_PF ahead.
__device__ __forceinline__ void dq_tile_full(const unsigned char* sK, const unsigned char* sV, const bf16x8 (&qf)[8],
                                             const bf16x8 (&gf)[8], const LaneOffs& lo_in, f32x16 (&dq)[4], float c2,
                                             float lse2, float Dq) {
    // the two offset registers are made opaque here so that the XORed per-block offsets are formed next
    // to each read (one vector op) instead of being kept in registers across the whole walk
    LaneOffs lo = lo_in;
    asm volatile("" : "+v"(lo.row), "+v"(lo.col));
    f32x16 s0, dp0, s1, dp1, zero;
#pragma unroll
    for (int i = 0; i < 16; ++i) zero[i] = 0.0f;
#define LRSA_DQ_OPND(n)                                                                                        \
    ((n) < 8 ? read_rows_o(sK, lo, 0, (n)) : (n) < 16 ? read_rows_o(sV, lo, 0, (n) - 8)                         \
     : (n) < 24 ? read_rows_o(sK, lo, 32, (n) - 16) : (n) < 32 ? read_rows_o(sV, lo, 32, (n) - 24)              \
     : read_cols_o(sK, lo, ((n) - 32) / 4 * 16, (n) & 3))
    bf16x8 a[DQ_PF];
#pragma unroll
    for (int n = 0; n < DQ_PF; ++n) a[n] = LRSA_DQ_OPND(n);
    const float neg_l = -lse2;
    bf16x8 dsf[4];   // dS of keys 0-15, 16-31, 32-47, 48-63
    // six groups of eight MFMAs (separate loops: each unrolls fully, so every array index is a constant)
#define LRSA_DQ_NEXT(n) if ((n) + DQ_PF < 48) a[(n) % DQ_PF] = LRSA_DQ_OPND((n) + DQ_PF)
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        s0 = mfma32(a[k % DQ_PF], qf[k], k == 0 ? zero : s0);
        LRSA_DQ_NEXT(k);
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        dp0 = mfma32(a[(8 + k) % DQ_PF], gf[k], k == 0 ? zero : dp0);
        LRSA_DQ_NEXT(8 + k);
#pragma unroll
        for (int i = 2 * k; i < 2 * k + 2; ++i) s0[i] = fast_exp2(__builtin_fmaf(s0[i], c2, neg_l));
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        s1 = mfma32(a[(16 + k) % DQ_PF], qf[k], k == 0 ? zero : s1);
        LRSA_DQ_NEXT(16 + k);
#pragma unroll
        for (int i = 2 * k; i < 2 * k + 2; ++i) s0[i] *= dp0[i] - Dq;
    }
    dsf[0] = pack8(s0, 0);
    dsf[1] = pack8(s0, 8);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        dp1 = mfma32(a[(24 + k) % DQ_PF], gf[k], k == 0 ? zero : dp1);
        LRSA_DQ_NEXT(24 + k);
#pragma unroll
        for (int i = 2 * k; i < 2 * k + 2; ++i) s1[i] = fast_exp2(__builtin_fmaf(s1[i], c2, neg_l));
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        dq[k & 3] = mfma32(a[(32 + k) % DQ_PF], dsf[k >> 2], dq[k & 3]);
        LRSA_DQ_NEXT(32 + k);
#pragma unroll
        for (int i = 2 * k; i < 2 * k + 2; ++i) s1[i] *= dp1[i] - Dq;
    }
    dsf[2] = pack8(s1, 0);
    dsf[3] = pack8(s1, 8);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        dq[k & 3] = mfma32(a[(40 + k) % DQ_PF], dsf[2 + (k >> 2)], dq[k & 3]);
        LRSA_DQ_NEXT(40 + k);
    }
#undef LRSA_DQ_NEXT
#undef LRSA_DQ_OPND
}

// GH query heads of one KV group share the workgroup (8 waves = GH heads x 256/GH queries), as in the forward.
// COMPACT: the rows of the gather list come from the condensed cache Kc, Vc (contiguous), no index is read.
template <int GH, bool COMPACT>
__global__ __launch_bounds__(DQ_THREADS, 2) void k_bwd_dq(Dims D, const bf16_t* __restrict__ Q,
                                                           const bf16_t* __restrict__ K,
                                                           const bf16_t* __restrict__ V,
                                                           const bf16_t* __restrict__ O,
                                                           const bf16_t* __restrict__ dO,
                                                           const float* __restrict__ lse,
                                                           float* __restrict__ Dsum, float* __restrict__ lse2_out,
                                                           const int32_t* __restrict__ idx,
                                                           const bf16_t* __restrict__ Kc,
                                                           const bf16_t* __restrict__ Vc,
                                                           bf16_t* __restrict__ dQ, QTileMap M) {
    constexpr int WPH = DQ_WAVES / GH;   // waves per head
    constexpr int QT = 32 * WPH;         // queries per head and workgroup
    __shared__ __attribute__((aligned(16))) unsigned char sK0[DQ_BN * TILE_ROW_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char sV0[DQ_BN * TILE_ROW_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char sK1[DQ_BN * TILE_ROW_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char sV1[DQ_BN * TILE_ROW_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    int b, h, gsub, tix;
    decode_qtile(M, D, blockIdx.x, b, h, gsub, tix);
    const int hq = h * D.G + gsub * GH + wave / WPH;
    const int wq = wave % WPH;

    int qc, t0, seg_end;
    if (tix < M.sink_tiles) {
        qc = -1; t0 = tix * QT; seg_end = D.S < D.n ? D.S : D.n;
    } else {
        const int tt = tix - M.sink_tiles;
        qc = tt / M.tpc;
        t0 = D.S + qc * D.L + (tt % M.tpc) * QT;
        const int64_t e = int64_t(D.S) + int64_t(qc + 1) * D.L;
        seg_end = e < D.n ? int(e) : D.n;
    }
    if (t0 >= seg_end) return;
    const int t_last = min(t0 + QT, seg_end) - 1;
    const int ng = gather_count(D, qc), cs = window_start(D, qc);
    const int m_max = ng + t_last - cs + 1;
    const int ntiles = (m_max + DQ_BN - 1) / DQ_BN;

    const bf16_t* Kh = K + b * D.ks[0] + h * D.ks[1];
    const bf16_t* Vh = V + b * D.ks[0] + h * D.ks[1];
    const int32_t* idx_h = idx + (int64_t(b) * D.Hkv + h) * D.Ns * D.K;

    const int tq = t0 + wq * 32 + l32;
    const int tq_ld = tq < t_last ? tq : t_last;
    const int64_t qoff = b * D.qs[0] + hq * D.qs[1] + int64_t(tq_ld) * D.qs[2];
    bf16x8 qf[8], gf[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        qf[kk] = *reinterpret_cast<const bf16x8*>(Q + qoff + kk * 16 + g * 8);
        gf[kk] = *reinterpret_cast<const bf16x8*>(dO + qoff + kk * 16 + g * 8);
    }
    // D = rowsum(dO * O) of this lane's row and its lse in log2 units: used here and, through the workspace,
    // by the key-outer kernel that runs after this one (every (head, query) row belongs to exactly one wave)
    const int64_t rowid = (int64_t(b) * D.Hq + hq) * D.lse_stride + tq_ld;
    const float lse2 = lse[rowid] * 1.4426950408889634f;
    float Dq = 0.0f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        const bf16x8 o8 = *reinterpret_cast<const bf16x8*>(O + qoff + kk * 16 + g * 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) Dq = __builtin_fmaf(float(o8[i]), float(gf[kk][i]), Dq);
    }
    Dq += __shfl_xor(Dq, 32, 64);
    if (tq <= t_last && g == 0) { Dsum[rowid] = -Dq; lse2_out[rowid] = lse2; }   // -D: the key-outer kernel starts its dA sums from it
    const int lim = ng + tq - cs;
    const int wave_lim_max = ng + min(t0 + wq * 32 + 31, t_last) - cs;

    const int64_t coff = COMPACT ? (int64_t(b) * D.Hkv + h) * (int64_t(D.S) + int64_t(D.K) * D.Ns) * 128 : 0;
    const bf16_t* Kc_h = Kc + coff;
    const bf16_t* Vc_h = Vc + coff;
    int pos[2];   // COMPACT: stream entries; else positions (fetched through idx one tile ahead)
    auto fetch_pos = [&](int tile) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int j = tile * DQ_BN + async_row(8 * wave + 4 * i, lane);
            j = j < m_max ? j : m_max - 1;
            pos[i] = COMPACT ? j : stream_pos(D, idx_h, j, ng, cs);
        }
    };
    auto issue = [&](unsigned char* sK, unsigned char* sV) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r4 = 8 * wave + 4 * i;
            const int ch = async_chunk(async_row(r4, lane), lane) * 8;
            if (COMPACT) {
                async_rows4(stream_row(Kc_h, Kh, D.ks[2], pos[i], ng, cs) + ch, sK, r4);
                async_rows4(stream_row(Vc_h, Vh, D.ks[2], pos[i], ng, cs) + ch, sV, r4);
            } else {
                const int64_t off = int64_t(pos[i]) * D.ks[2] + ch;
                async_rows4(Kh + off, sK, r4);
                async_rows4(Vh + off, sV, r4);
            }
        }
    };

    const float c2 = D.scale * 1.4426950408889634f;
    const LaneOffs lo = make_lane_offs(lane);
    const int wave_lim_min = ng + t0 + wq * 32 - cs;   // last stream entry the wave's first query sees
#define LRSA_DQ_TILE(sK, sV, j0_)                                                                              \
    {                                                                                                           \
        const int j0 = (j0_);                                                                                   \
        if (j0 + DQ_BN - 1 <= wave_lim_min)                                                                     \
            dq_tile_full(sK, sV, qf, gf, lo, dq, c2, lse2, Dq);                                                 \
        else if (j0 <= wave_lim_max)                                                                            \
            dq_tile<true>(sK, sV, qf, gf, lo, dq, j0, lim, wave_lim_max, c2, lse2, Dq, lane);                   \
    }
    f32x16 dq[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dq[db][i] = 0.0f;

    fetch_pos(0);
    issue(sK0, sV0);
    if (ntiles > 1) fetch_pos(1);
    for (int tile = 0; tile < ntiles; tile += 2) {
        wait_vmcnt<0>();
        __syncthreads();
        if (tile + 1 < ntiles) {
            issue(sK1, sV1);
            if (tile + 2 < ntiles) fetch_pos(tile + 2);
        }
        LRSA_DQ_TILE(sK0, sV0, tile * DQ_BN);
        if (tile + 1 >= ntiles) break;
        wait_vmcnt<0>();
        __syncthreads();
        if (tile + 2 < ntiles) {
            issue(sK0, sV0);
            if (tile + 3 < ntiles) fetch_pos(tile + 3);
        }
        LRSA_DQ_TILE(sK1, sV1, (tile + 1) * DQ_BN);
    }

#undef LRSA_DQ_TILE

    if (tq <= t_last) {
        bf16_t* orow = dQ + b * D.qs[0] + hq * D.qs[1] + int64_t(tq) * D.qs[2];
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                f32x4 v;
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = dq[db][a * 4 + r] * D.scale;
                *reinterpret_cast<bf16x4*>(orow + db * 32 + a * 8 + g * 4) = __builtin_convertvector(v, bf16x4);
            }
    }
}

// ------------------------------------------------------------------------------------ dK, dV
// first query chunk that sees entry j0 of the gather list
__device__ __forceinline__ int first_chunk_seeing(const Dims& D, int j0) {
    return j0 < D.S ? 0 : (j0 - D.S) / D.K + D.lp + 1;
}

// One sub-step (32 query rows: rows rowbase .. rowbase+31 of the stage tiles) of the key-outer walk for
// one wave.  sLD holds this wave's copy of the stage rows' lse in log2 units (floats 0..KV_ROWS-1) and -D
// (the next KV_ROWS floats; D = rowsum(dO * O), negated by the query-outer kernel that wrote it).  r0 = first row of the sub-step; rows >= tb are padding.
// lim_u: GATHER (steps never straddle a chunk): the largest gather-list entry the step's chunk sees.
// The wave's K fragments are in registers, its V rows in LDS (sVw): K fragments and the accumulators
// fill the register file.
template <bool GATHER>
__device__ __forceinline__ void dkv_step(const Dims& D, const unsigned char* sQ, const unsigned char* sG,
                                         const float* sLD, const bf16x8 (&kf)[KV_NB][8], const unsigned char* sVw,
                                         const LaneOffs& lo_in, f32x16 (&dk)[KV_NB][4], f32x16 (&dv)[KV_NB][4], int r0,
                                         int tb, const int (&kcmp)[KV_NB], int lim_u, bool need_mask, float c2, int lane,
                                         int rowbase) {
    const int g = lane >> 5;
    // the two offset registers are made opaque here so that the XORed per-block offsets are formed next
    // to each read (one VALU op) instead of being kept in sixteen registers across the whole walk
    // The lane's offsets with the addresses of the three tiles folded in (the tiles start on 256-byte
    // boundaries): one add per tile and sub-step, then one XOR per read.  The registers are made opaque so
    // that the XORed per-block addresses are formed next to each read instead of being kept across the walk.
    unsigned aQr = lo_in.row + lds_addr(sQ) + rowbase * TILE_ROW_BYTES, aQc = lo_in.col + lds_addr(sQ) + rowbase * TILE_ROW_BYTES;
    unsigned aGr = lo_in.row + lds_addr(sG) + rowbase * TILE_ROW_BYTES, aGc = lo_in.col + lds_addr(sG) + rowbase * TILE_ROW_BYTES;
    unsigned aVr = lo_in.row + lds_addr(sVw);
    asm volatile("" : "+v"(aQr), "+v"(aQc), "+v"(aGr), "+v"(aGc), "+v"(aVr));
    // Four MFMA groups: S, dA, dV, dK (8 MFMAs per 32-key block each).  The vector work between them is
    // written next to MFMAs it does not depend on -- exp(S) beside the dA group, dS beside the dV group --
    // so that one wave keeps both pipes busy.  Operands are read two ahead of the MFMAs that consume them;
    // an operand read from the Q / dO stage serves all key blocks of the wave.
    bf16x8 a[2];
    f32x16 s[KV_NB], dp[KV_NB];
    // dA - D comes out of the MFMAs themselves: the accumulators start from -D of their rows (sLD holds -D)
#pragma unroll
    for (int a4 = 0; a4 < 4; ++a4) {
        const f32x4 d4 = *reinterpret_cast<const f32x4*>(sLD + KV_ROWS + rowbase + 8 * a4 + 4 * g);
#pragma unroll
        for (int nb = 0; nb < KV_NB; ++nb)
#pragma unroll
            for (int r = 0; r < 4; ++r) dp[nb][a4 * 4 + r] = d4[r];
    }
#pragma unroll
    for (int nb = 0; nb < KV_NB; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[nb][i] = 0.0f;
    a[0] = read_rows_a(aQr, 0);
    a[1] = read_rows_a(aQr, 1);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
#pragma unroll
        for (int nb = 0; nb < KV_NB; ++nb) s[nb] = mfma32(a[kk & 1], kf[nb][kk], s[nb]);
        a[kk & 1] = kk < 6 ? read_rows_a(aQr, kk + 2) : read_rows_a(aGr, kk - 6);
    }
    // mask bounds: row rho = 8*a4 + 4g + r of the step is visible to key block nb iff mlo[nb] <= 8*a4 + r < mhi
    const int mhi = (tb - r0) - 4 * g;
    int mlo[KV_NB];
#pragma unroll
    for (int nb = 0; nb < KV_NB; ++nb)
        mlo[nb] = GATHER ? (kcmp[nb] <= lim_u ? -64 : 64) : (kcmp[nb] == 0x7fffffff ? 64 : kcmp[nb] - r0 - 4 * g);
    // A = exp2(S*c2 - lse2), four values per key block and pair of MFMA rounds; sLD holds lse already in
    // log2 units.  Only steps that touch the diagonal, a partly visible gather prefix, padding rows or
    // padding keys pay for the mask (wave-uniform flag).
    bf16x8 vb[KV_NB][2];
#pragma unroll
    for (int nb = 0; nb < KV_NB; ++nb) vb[nb][0] = read_rows_a(aVr + nb * 32 * TILE_ROW_BYTES, 0);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
#pragma unroll
        for (int nb = 0; nb < KV_NB; ++nb) {
            if (kk + 1 < 8) vb[nb][(kk + 1) & 1] = read_rows_a(aVr + nb * 32 * TILE_ROW_BYTES, kk + 1);
            dp[nb] = mfma32(a[kk & 1], vb[nb][kk & 1], dp[nb]);
        }
        // next operands: the rest of the dO rows, then the first transposed dO operands
        if (kk < 6) a[kk & 1] = read_rows_a(aGr, kk + 2);
        else a[kk & 1] = read_cols_a(aGc, 0, kk - 6);
        if ((kk & 1) == 0) {
            const int a4 = kk >> 1;
            const f32x4 l4 = *reinterpret_cast<const f32x4*>(sLD + rowbase + 8 * a4 + 4 * g);
            if (!need_mask) {
#pragma unroll
                for (int nb = 0; nb < KV_NB; ++nb)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        s[nb][a4 * 4 + r] = fast_exp2(__builtin_fmaf(s[nb][a4 * 4 + r], c2, -l4[r]));
            } else {
#pragma unroll
                for (int nb = 0; nb < KV_NB; ++nb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float pr = fast_exp2(__builtin_fmaf(s[nb][a4 * 4 + r], c2, -l4[r]));
                        const int c = 8 * a4 + r;
                        s[nb][a4 * 4 + r] = (c >= mlo[nb] && c < mhi) ? pr : 0.0f;
                    }
            }
        }
    }
    bf16x8 pf[KV_NB][2], dsf[KV_NB][2];
#pragma unroll
    for (int nb = 0; nb < KV_NB; ++nb) { pf[nb][0] = pack8(s[nb], 0); pf[nb][1] = pack8(s[nb], 8); }
    // dV^T += dO^T A (rows 0-15 blocks 0..3, rows 16-31 blocks 0..3) with dS = A * (dA - D) beside it (dp holds dA - D),
    // then dK^T += Q^T dS in the same order
#define LRSA_OPND(n) ((n) < 8 ? read_cols_a(aGc, ((n) >> 2) * 16, (n) & 3) : read_cols_a(aQc, (((n) - 8) >> 2) * 16, (n) & 3))
#pragma unroll
    for (int n = 0; n < 8; ++n) {
#pragma unroll
        for (int nb = 0; nb < KV_NB; ++nb) dv[nb][n & 3] = mfma32(a[n & 1], pf[nb][n >> 2], dv[nb][n & 3]);
        a[n & 1] = LRSA_OPND(n + 2);
        if ((n & 1) == 0) {
            const int a4 = n >> 1;
#pragma unroll
            for (int nb = 0; nb < KV_NB; ++nb)
#pragma unroll
                for (int r = 0; r < 4; ++r) dp[nb][a4 * 4 + r] *= s[nb][a4 * 4 + r];
        }
    }
#pragma unroll
    for (int nb = 0; nb < KV_NB; ++nb) { dsf[nb][0] = pack8(dp[nb], 0); dsf[nb][1] = pack8(dp[nb], 8); }
#pragma unroll
    for (int n = 8; n < 16; ++n) {
#pragma unroll
        for (int nb = 0; nb < KV_NB; ++nb) dk[nb][n & 3] = mfma32(a[n & 1], dsf[nb][(n - 8) >> 2], dk[nb][n & 3]);
        if (n + 2 < 16) a[n & 1] = LRSA_OPND(n + 2);
    }
#undef LRSA_OPND
}

// Two stages of 64 rows: one barrier per 64 MFMAs of a wave; the copies of the next stage run during
// the two sub-steps of the current one.

// LDS of the dK/dV kernel: two stages of (Q rows, dO rows, per-wave lse|D) -- separate arrays so that reads
// of one stage need not wait for the asynchronous fill of the other -- and the workgroup's V rows
struct KvLds {
    unsigned char *sQ0, *sQ1, *sG0, *sG1;
    float *sL0, *sL1;
    unsigned char* sVk;
};
// one set of arrays for both instantiations of the body (a template would get a set each)
__device__ __forceinline__ KvLds kv_lds() {
    __shared__ __attribute__((aligned(256))) unsigned char sQ0[KV_ROWS * TILE_ROW_BYTES], sQ1[KV_ROWS * TILE_ROW_BYTES];
    __shared__ __attribute__((aligned(256))) unsigned char sG0[KV_ROWS * TILE_ROW_BYTES], sG1[KV_ROWS * TILE_ROW_BYTES];
    __shared__ __attribute__((aligned(16))) float sL0[KV_WAVES * 2 * KV_ROWS], sL1[KV_WAVES * 2 * KV_ROWS];
    __shared__ __attribute__((aligned(256))) unsigned char sVk[KV_BK * TILE_ROW_BYTES];
    return KvLds{sQ0, sQ1, sG0, sG1, sL0, sL1, sVk};
}

template <bool GATHER>
__device__ __forceinline__ void dkv_body(const Dims& D, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                                         const bf16_t* __restrict__ V, const bf16_t* __restrict__ Kc,
                                         const bf16_t* __restrict__ Vc, const bf16_t* __restrict__ dO,
                                         const float* __restrict__ lse, const float* __restrict__ Dsum,
                                         const int32_t* __restrict__ idx, bf16_t* __restrict__ dK,
                                         bf16_t* __restrict__ dV, float* __restrict__ accK, float* __restrict__ accV,
                                         float* __restrict__ part, const BwdPlan& P, const int block) {
    const KvLds sh = kv_lds();
    unsigned char *const sQ0 = sh.sQ0, *const sQ1 = sh.sQ1, *const sG0 = sh.sG0, *const sG1 = sh.sG1;
    float *const sL0 = sh.sL0, *const sL1 = sh.sL1;
    unsigned char* const sVk = sh.sVk;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: kept in a scalar register
    const int l32 = lane & 31, g = lane >> 5;
    // ---- which keys, which query rows.  The grid is one-dimensional and workgroup i runs on XCD i % 8
    // (each XCD has its own L2).  GATHER: all list tiles of one (batch, KV head, query slice) stream the
    // same Q and dO rows; they get consecutive slots of ONE XCD, so those rows are fetched from memory once
    // per XCD, not once per tile.  WINDOW: tiles in position order, latest first, spread over the XCDs.
    int key0, key_end;   // key ids of this workgroup: positions (WINDOW) or gather-list entries (GATHER)
    int ta, tb;          // query rows [ta, tb) of every head of the group
    int qa = 0;          // GATHER: first query chunk of the slice
    int slice = 0;
    int unit;
    {
        const int xcd = block & 7, seq = block >> 3;
        if (GATHER) {
            const int grp = xcd + 8 * (seq / P.gtiles);
            const int units = D.B * D.Hkv;
            if (grp >= units * P.nsl) return;
            unit = grp % units;
            slice = P.nsl - 1 - grp / units;          // latest slices (most list tiles) first
            key0 = (seq % P.gtiles) * KV_BK;
        } else {
            unit = block / P.ktiles;
            key0 = P.ktiles - 1 - block % P.ktiles;   // tile index for now
        }
    }
    const int h = unit % D.Hkv, b = unit / D.Hkv;
    const int32_t* idx_h = idx + (int64_t(b) * D.Hkv + h) * D.Ns * D.K;
    if (GATHER) {
        // slice = query chunks [slice*qch, (slice+1)*qch), of which the tile sees those from qf on
        key_end = P.gl_total;
        const int qf = first_chunk_seeing(D, key0);
        qa = max(P.fq0 + slice * P.qch, qf);
        const int qb = min(P.fq1, P.fq0 + (slice + 1) * P.qch);
        if (qa >= qb) return;
        ta = D.S + qa * D.L;
        const int64_t e = int64_t(D.S) + int64_t(qb) * D.L;
        tb = e < D.n ? int(e) : D.n;
    } else {
        const int tix = key0;
        if (tix < P.sink_tiles_k) {
            key0 = tix * KV_BK;
            key_end = D.S < D.n ? D.S : D.n;
            tb = key_end < D.row_end ? key_end : D.row_end;   // only sink queries see sink keys through the window
        } else {
            const int tt = tix - P.sink_tiles_k;
            const int kc = P.kc_lo + tt / P.tpc_k;
            key0 = D.S + kc * D.L + (tt % P.tpc_k) * KV_BK;
            const int64_t e = int64_t(D.S) + int64_t(kc + 1) * D.L;
            key_end = e < D.n ? int(e) : D.n;
            const int64_t e2 = int64_t(D.S) + (int64_t(kc) + 1 + D.lp) * D.L;
            tb = e2 < D.row_end ? int(e2) : D.row_end;
        }
        if (key0 >= key_end) return;
        ta = key0 > D.row_begin ? key0 : D.row_begin;
        if (ta >= tb) return;
    }
    // Steps of KV_ROWS rows.  WINDOW: consecutive rows of [ta, tb).  GATHER: chunk by chunk (the last step
    // of a chunk may be partial), so that one step never sees two different gather-list prefixes.
    const int spc = (D.L + KV_ROWS - 1) / KV_ROWS;                               // GATHER: steps per chunk
    const int sph = GATHER ? ((tb - ta + D.L - 1) / D.L) * spc : (tb - ta + KV_ROWS - 1) / KV_ROWS;   // steps per head
    const int nsteps = sph * D.G;
    // first row, row end and chunk-visible limit of a step
    auto step_rows = [&](int sidx, int& r0, int& rend, int& lim_u) {
        const int w = sidx % sph;
        if (GATHER) {
            const int c = qa + w / spc;
            r0 = D.S + c * D.L + (w % spc) * KV_ROWS;
            const int64_t e = int64_t(D.S) + int64_t(c + 1) * D.L;
            rend = e < tb ? int(e) : tb;
            lim_u = gather_count(D, c) - 1;
        } else {
            r0 = ta + w * KV_ROWS;
            rend = tb;
            lim_u = 0;
        }
    };

    // ---- this lane's key columns (one per 32-key block): K fragments stay in registers, the V rows
    // go to LDS in the swizzled tile layout (row = key within the workgroup)
    const int wave_key0 = key0 + wave * (32 * KV_NB);
    const bool wave_keys_valid = wave_key0 + 32 * KV_NB - 1 < key_end;
    int kcmp[KV_NB];
    bf16x8 kf[KV_NB][8];
#pragma unroll
    for (int nb = 0; nb < KV_NB; ++nb) {
        const int kidn = wave_key0 + nb * 32 + l32;
        const bool kvalid = kidn < key_end;
        const int kid_ld = kvalid ? kidn : key_end - 1;
        kcmp[nb] = kvalid ? kidn : 0x7fffffff;
        // the key's K and V rows: by position, or (GATHER with a condensed cache) row kid of the contiguous copy
        const bf16_t *krow, *vrow_src;
        if (GATHER && D.compact) {
            const int64_t coff = ((int64_t(b) * D.Hkv + h) * P.gl_total + kid_ld) * 128;
            krow = Kc + coff;
            vrow_src = Vc + coff;
        } else {
            const int kpos = GATHER ? (kid_ld < D.S ? kid_ld : idx_h[kid_ld - D.S]) : kid_ld;
            const int64_t koff = b * D.ks[0] + h * D.ks[1] + int64_t(kpos) * D.ks[2];
            krow = K + koff;
            vrow_src = V + koff;
        }
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) kf[nb][kk] = *reinterpret_cast<const bf16x8*>(krow + kk * 16 + g * 8);
        const int vrow = wave * (32 * KV_NB) + nb * 32 + l32;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
            *reinterpret_cast<bf16x8*>(sVk + tile_off(vrow, kk * 2 + g)) =
                *reinterpret_cast<const bf16x8*>(vrow_src + kk * 16 + g * 8);
    }
    const unsigned char* sVw = sVk + wave * (32 * KV_NB) * TILE_ROW_BYTES;
    const LaneOffs lo = make_lane_offs(lane);

    // ---- loader: wave w fills rows 8w .. 8w+7 of the Q and dO tiles (two copies of 4 rows each) and
    // its own lse|D block (one copy each).
    auto issue = [&](int step, unsigned char* sQ, unsigned char* sG, float* sL) {
        const int gi = step / sph;
        int r0, rend, lim_unused;
        step_rows(step, r0, rend, lim_unused);
        const int hq = h * D.G + gi;
        const int64_t base = b * D.qs[0] + hq * D.qs[1];
#pragma unroll
        for (int i = 0; i < KV_ROWS / (4 * KV_WAVES); ++i) {
            const int r4 = (KV_ROWS / KV_WAVES) * wave + 4 * i;
            const int row = async_row(r4, lane);
            const int t = min(r0 + row, rend - 1);
            const int64_t off = base + int64_t(t) * D.qs[2] + async_chunk(row, lane) * 8;
            async_rows4(Q + off, sQ, r4);
            async_rows4(dO + off, sG, r4);
        }
        const int64_t rid = (int64_t(b) * D.Hq + hq) * D.lse_stride + min(r0 + lane, rend - 1);
        async_copy4(lse + rid, sL + wave * 2 * KV_ROWS);
        async_copy4(Dsum + rid, sL + wave * 2 * KV_ROWS + KV_ROWS);
    };

    const float c2 = D.scale * 1.4426950408889634f;
    f32x16 dk[KV_NB][4], dv[KV_NB][4];
#pragma unroll
    for (int nb = 0; nb < KV_NB; ++nb)
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) { dk[nb][db][i] = 0.0f; dv[nb][db][i] = 0.0f; }

#define LRSA_KV_STEP(step, sQ, sG, sL, sQn, sGn, sLn)                                                   \
    {                                                                                                    \
        wait_vmcnt<0>();     /* this wave's copies for `step` have landed */                             \
        __syncthreads();     /* ... everybody's have, and everybody is done with the other stage */      \
        if ((step) + 1 < nsteps) issue((step) + 1, sQn, sGn, sLn);                                       \
        int r0s_, rend_, lim_u_;                                                                         \
        step_rows(step, r0s_, rend_, lim_u_);                                                            \
        _Pragma("unroll 1") for (int sub_ = 0; sub_ < KV_SUB; ++sub_) {                                    \
            const int r0_ = r0s_ + sub_ * KV_BQ;                                                         \
            /* nothing to do: padding rows only, or (WINDOW) rows before the wave's first key.  The flag */ \
            /* is made opaque so that each sub-step body stays a basic block of its own: merged into one */ \
            /* block the bodies get interleaved and the register file overflows.                        */ \
            int run_ = (r0_ < rend_ && (GATHER || r0_ + KV_BQ - 1 >= wave_key0)) ? 1 : 0;                \
            run_ = __builtin_amdgcn_readfirstlane(run_); /* wave-uniform by construction */              \
            asm volatile("" : "+s"(run_));                                                               \
            /* every (row, key) pair of the sub-step visible for this wave? */                           \
            const bool full_ = wave_keys_valid && r0_ + KV_BQ <= rend_ &&                                \
                               (GATHER ? lim_u_ >= wave_key0 + 32 * KV_NB - 1 : r0_ >= wave_key0 + 32 * KV_NB - 1); \
            if (run_)                                                                                    \
                dkv_step<GATHER>(D, sQ, sG, sL + wave * 2 * KV_ROWS, kf, sVw, lo, dk, dv, r0_, rend_, kcmp, lim_u_, \
                                 !full_, c2, lane, sub_ * KV_BQ);                                        \
        }                                                                                                \
    }

    // the K fragments have arrived before the first asynchronous copy is issued: the compiler then places
    // no vector-memory waits of its own in the loop (they would also wait for the copies in flight)
    wait_all_vmem_known();
#pragma unroll
    for (int nb = 0; nb < KV_NB; ++nb)
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) pin_loaded(kf[nb][kk]);
    issue(0, sQ0, sG0, sL0);
    for (int step = 0; step < nsteps; step += 2) {
        LRSA_KV_STEP(step, sQ0, sG0, sL0, sQ1, sG1, sL1);
        if (step + 1 >= nsteps) break;
        LRSA_KV_STEP(step + 1, sQ1, sG1, sL1, sQ0, sG0, sL0);
    }
#undef LRSA_KV_STEP

    const size_t part_stride = size_t(D.B) * D.Hkv * P.gl_total * 128;   // floats per slice
    const size_t part_v = size_t(P.nsl + 1) * part_stride;                // dV partials follow the dK partials
#pragma unroll
    for (int nb = 0; nb < KV_NB; ++nb) {
        const int kidn = key0 + wave * (32 * KV_NB) + nb * 32 + (lane & 31);
        if (kidn >= key_end) continue;
        if (GATHER) {
            float* pk = part + size_t(slice) * part_stride + ((size_t(b) * D.Hkv + h) * P.gl_total + kidn) * 128;
            float* pv = pk + part_v;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    f32x4 x, y;
#pragma unroll
                    for (int r = 0; r < 4; ++r) { x[r] = dk[nb][db][a * 4 + r] * D.scale; y[r] = dv[nb][db][a * 4 + r]; }
                    *reinterpret_cast<f32x4*>(pk + db * 32 + a * 8 + g * 4) = x;
                    *reinterpret_cast<f32x4*>(pv + db * 32 + a * 8 + g * 4) = y;
                }
        } else {
            // gather-list entry of this position, if it is a sink token or a survivor
            int j = -1;
            if (P.gtiles > 0) {
                if (kidn < D.S) j = kidn;
                else {
                    const int c = (kidn - D.S) / D.L;
                    if (D.S + (c + 1) * D.K <= P.gl_total) {   // chunk c is compressed for some query of this call
                        const int32_t* rowp = idx_h + int64_t(c) * D.K;
                        int lo_ = 0, hi_ = D.K - 1;
                        while (lo_ <= hi_) {
                            const int mid = (lo_ + hi_) >> 1;
                            const int v = rowp[mid];
                            if (v == kidn) { j = D.S + c * D.K + mid; break; }
                            if (v < kidn) lo_ = mid + 1; else hi_ = mid - 1;
                        }
                    }
                }
            }
            const int64_t koff = b * D.ks[0] + h * D.ks[1] + int64_t(kidn) * D.ks[2];
            // listed positions: fp32 into the extra slot, the reduction kernel adds the slices; others: final
            float* pk = j >= 0 ? part + size_t(P.nsl) * part_stride + ((size_t(b) * D.Hkv + h) * P.gl_total + j) * 128 : nullptr;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    f32x4 x, y;
#pragma unroll
                    for (int r = 0; r < 4; ++r) { x[r] = dk[nb][db][a * 4 + r] * D.scale; y[r] = dv[nb][db][a * 4 + r]; }
                    const int dcol = db * 32 + a * 8 + g * 4;
                    if (j >= 0) {
                        *reinterpret_cast<f32x4*>(pk + dcol) = x;
                        *reinterpret_cast<f32x4*>(pk + part_v + dcol) = y;
                    } else if (D.acc) {
                        // row window: this call's share is added to the caller's fp32 sums (one writer per element)
                        const int64_t aoff = ((int64_t(b) * D.Hkv + h) * D.n + kidn) * 128 + dcol;
                        *reinterpret_cast<f32x4*>(accK + aoff) += x;
                        *reinterpret_cast<f32x4*>(accV + aoff) += y;
                    } else {
                        *reinterpret_cast<bf16x4*>(dK + koff + dcol) = __builtin_convertvector(x, bf16x4);
                        *reinterpret_cast<bf16x4*>(dV + koff + dcol) = __builtin_convertvector(y, bf16x4);
                    }
                }
        }
    }
}

// One launch for all of dK/dV: the GATHER workgroups first (equal, long), then the WINDOW workgroups, so that
// the chip has one tail, not two.
__global__ __launch_bounds__(KV_THREADS, KV_WAVES == 8 ? 2 : 1) void k_bwd_dkv(Dims D, const bf16_t* __restrict__ Q,
                                                                                const bf16_t* __restrict__ K,
                                                                                const bf16_t* __restrict__ V,
                                                                                const bf16_t* __restrict__ Kc,
                                                                                const bf16_t* __restrict__ Vc,
                                                                                const bf16_t* __restrict__ dO,
                                                                                const float* __restrict__ lse,
                                                                                const float* __restrict__ Dsum,
                                                                                const int32_t* __restrict__ idx,
                                                                                bf16_t* __restrict__ dK,
                                                                                bf16_t* __restrict__ dV,
                                                                                float* __restrict__ accK,
                                                                                float* __restrict__ accV,
                                                                                float* __restrict__ part, BwdPlan P) {
    const int block = blockIdx.x;
    if (block < P.gather_wgs) dkv_body<true>(D, Q, K, V, Kc, Vc, dO, lse, Dsum, idx, dK, dV, accK, accV, part, P, block);
    else dkv_body<false>(D, Q, K, V, Kc, Vc, dO, lse, Dsum, idx, dK, dV, accK, accV, part, P, block - P.gather_wgs);
}

// dK, dV of the listed positions (sink tokens and survivors): the WINDOW contribution plus the GATHER slices
// that exist for the entry's list tile, added in a fixed order.  32 threads per entry, 4 channels each.
__global__ __launch_bounds__(256) void k_bwd_dkv_reduce(Dims D, const int32_t* __restrict__ idx,
                                                        const float* __restrict__ part, bf16_t* __restrict__ dK,
                                                        bf16_t* __restrict__ dV, float* __restrict__ accK,
                                                        float* __restrict__ accV, float* __restrict__ dKc,
                                                        float* __restrict__ dVc, BwdPlan P) {
    const int64_t e = int64_t(blockIdx.x) * 8 + (threadIdx.x >> 5);   // (b, h, entry)
    const int64_t total = int64_t(D.B) * D.Hkv * P.gl_total;
    if (e >= total) return;
    const int j = int(e % P.gl_total);
    const int bh = int(e / P.gl_total);
    const int b = bh / D.Hkv, h = bh % D.Hkv;
    const int pos = j < D.S ? j : idx[(int64_t(bh) * D.Ns) * D.K + (j - D.S)];
    const size_t part_stride = size_t(D.B) * D.Hkv * P.gl_total * 128;
    const size_t part_v = size_t(P.nsl + 1) * part_stride;
    const int dcol = (threadIdx.x & 31) * 4;
    const float* p0 = part + size_t(e) * 128 + dcol;
    f32x4 x = {0.0f, 0.0f, 0.0f, 0.0f}, y = {0.0f, 0.0f, 0.0f, 0.0f};
    // the WINDOW workgroups of this call cover the sink (with a row window: only when its rows are in it) and the
    // key chunks from kc_lo on
    const bool in_window = pos < D.S ? P.sink_tiles_k > 0 : (pos - D.S) / D.L >= P.kc_lo;
    if (in_window) {
        x = *reinterpret_cast<const f32x4*>(p0 + size_t(P.nsl) * part_stride);
        y = *reinterpret_cast<const f32x4*>(p0 + size_t(P.nsl) * part_stride + part_v);
    }
    const int qf0 = first_chunk_seeing(D, (j / KV_BK) * KV_BK);
    if (qf0 < P.fq1)
        for (int sl = qf0 > P.fq0 ? (qf0 - P.fq0) / P.qch : 0; sl < P.nsl; ++sl) {
            x += *reinterpret_cast<const f32x4*>(p0 + size_t(sl) * part_stride);
            y += *reinterpret_cast<const f32x4*>(p0 + size_t(sl) * part_stride + part_v);
        }
    if (D.acc) {
        const int64_t aoff = ((int64_t(b) * D.Hkv + h) * D.n + pos) * 128 + dcol;
        *reinterpret_cast<f32x4*>(accK + aoff) += x;
        *reinterpret_cast<f32x4*>(accV + aoff) += y;
        return;
    }
    if (dKc) {   // condensed cache: the gradient of the condensed rows is a product of its own, scattered afterwards
        *reinterpret_cast<f32x4*>(dKc + e * 128 + dcol) = x;
        *reinterpret_cast<f32x4*>(dVc + e * 128 + dcol) = y;
        return;
    }
    const int64_t koff = b * D.ks[0] + h * D.ks[1] + int64_t(pos) * D.ks[2];
    *reinterpret_cast<bf16x4*>(dK + koff + dcol) = __builtin_convertvector(x, bf16x4);
    *reinterpret_cast<bf16x4*>(dV + koff + dcol) = __builtin_convertvector(y, bf16x4);
}

// Condensed cache: dKc, dVc [B, Hkv, gl, 128] fp32 -> rows of dK, dV at the positions of the gather list.  Every
// position occurs once in the list, so the scatter has no collisions and needs no addition.
__global__ __launch_bounds__(256) void k_bwd_scatter_dkv(Dims D, const int32_t* __restrict__ idx,
                                                         const float* __restrict__ dKc, const float* __restrict__ dVc,
                                                         bf16_t* __restrict__ dK, bf16_t* __restrict__ dV, int gl) {
    const int64_t e = int64_t(blockIdx.x) * 8 + (threadIdx.x >> 5);   // (b, h, entry)
    if (e >= int64_t(D.B) * D.Hkv * gl) return;
    const int j = int(e % gl), bh = int(e / gl);
    const int b = bh / D.Hkv, h = bh % D.Hkv;
    const int pos = j < D.S ? j : idx[(int64_t(bh) * D.Ns) * D.K + (j - D.S)];
    const int dcol = (threadIdx.x & 31) * 4;
    const int64_t koff = b * D.ks[0] + h * D.ks[1] + int64_t(pos) * D.ks[2];
    *reinterpret_cast<bf16x4*>(dK + koff + dcol) = __builtin_convertvector(*reinterpret_cast<const f32x4*>(dKc + e * 128 + dcol), bf16x4);
    *reinterpret_cast<bf16x4*>(dV + koff + dcol) = __builtin_convertvector(*reinterpret_cast<const f32x4*>(dVc + e * 128 + dcol), bf16x4);
}

// fp32 sums of a sequence of row-window calls -> dK, dV in the tensors' dtype (32 lanes per row)
__global__ __launch_bounds__(256) void k_bwd_acc_finish(Dims D, const float* __restrict__ accK,
                                                        const float* __restrict__ accV, bf16_t* __restrict__ dK,
                                                        bf16_t* __restrict__ dV) {
    const int64_t e = int64_t(blockIdx.x) * 8 + (threadIdx.x >> 5);   // (b, h, position)
    if (e >= int64_t(D.B) * D.Hkv * D.n) return;
    const int pos = int(e % D.n), bh = int(e / D.n);
    const int b = bh / D.Hkv, h = bh % D.Hkv;
    const int dcol = (threadIdx.x & 31) * 4;
    const f32x4 x = *reinterpret_cast<const f32x4*>(accK + e * 128 + dcol);
    const f32x4 y = *reinterpret_cast<const f32x4*>(accV + e * 128 + dcol);
    const int64_t koff = b * D.ks[0] + h * D.ks[1] + int64_t(pos) * D.ks[2];
    *reinterpret_cast<bf16x4*>(dK + koff + dcol) = __builtin_convertvector(x, bf16x4);
    *reinterpret_cast<bf16x4*>(dV + koff + dcol) = __builtin_convertvector(y, bf16x4);
}

hipError_t launch_bwd_acc_finish(const Dims& D, const float* accK, const float* accV, void* dK, void* dV, hipStream_t st) {
    const int64_t rows = int64_t(D.B) * D.Hkv * D.n;
    LRSA_TIMED_LAUNCH("k_bwd_acc_finish", st, k_bwd_acc_finish, dim3((unsigned)((rows + 7) / 8)), dim3(256), 0, st, D, accK,
                      accV, (bf16_t*)dK, (bf16_t*)dV);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ launcher
hipError_t launch_attn_bwd_mfma(const Dims& D, const void* Q, const void* K, const void* V, const void* O,
                                const void* dO, const float* lse, const int32_t* idx, void* dQ, void* dK,
                                void* dV, float* accK, float* accV, void* ws, hipStream_t st) {
    const BwdPlan P = make_plan(D);
    // D and lse in log2 units hold the rows of the window only; like the caller's tensors they are addressed by
    // absolute row, hence the shifted bases
    float* Dsum = reinterpret_cast<float*>(ws) - D.row_begin;
    float* lse2 = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + P.off_lse2) - D.row_begin;
    float* part = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + P.off_part);
    const bf16_t *q = (const bf16_t*)Q, *k = (const bf16_t*)K, *v = (const bf16_t*)V, *o = (const bf16_t*)O,
                 *g = (const bf16_t*)dO;

    const bool compact = D.compact && P.gl_total > 0;
    const bf16_t *kc = nullptr, *vc = nullptr;
    {
        const int gh = heads_per_wg(D);
        const QTileMap M = make_qtile_map(D, gh, DQ_WAVES);
        const int64_t wgs = int64_t(D.B) * D.Hkv * M.per_unit;
        if (compact && wgs > 0) {
            kc = reinterpret_cast<const bf16_t*>(reinterpret_cast<const char*>(ws) + P.off_compact);
            vc = reinterpret_cast<const bf16_t*>(reinterpret_cast<const char*>(ws) + P.off_compact + compact_kv_bytes(D) / 2);
            const hipError_t e = launch_compact_kv(D, K, V, idx, (void*)kc, (void*)vc, st);
            if (e != hipSuccess) return e;
        }
#define LRSA_DQ_LAUNCH(GH_, C_)                                                                                     \
    LRSA_TIMED_LAUNCH("k_bwd_dq", st, (k_bwd_dq<GH_, C_>), dim3((unsigned)wgs), dim3(DQ_THREADS), 0, st, D, q, k, v, o, g, lse, \
                      Dsum, lse2, idx, kc, vc, (bf16_t*)dQ, M)
        if (wgs > 0) {
            if (gh == 4) { if (compact) LRSA_DQ_LAUNCH(4, true); else LRSA_DQ_LAUNCH(4, false); }
            else if (gh == 2) { if (compact) LRSA_DQ_LAUNCH(2, true); else LRSA_DQ_LAUNCH(2, false); }
            else { if (compact) LRSA_DQ_LAUNCH(1, true); else LRSA_DQ_LAUNCH(1, false); }
        }
#undef LRSA_DQ_LAUNCH
    }
    const int64_t wgs = int64_t(P.gather_wgs) + int64_t(D.B) * D.Hkv * P.ktiles;
    if (wgs > 0)
        LRSA_TIMED_LAUNCH("k_bwd_dkv", st, k_bwd_dkv, dim3((unsigned)wgs), dim3(KV_THREADS), 0, st, D, q, k, v, kc, vc, g,
                          lse2, Dsum, idx, (bf16_t*)dK, (bf16_t*)dV, accK, accV, part, P);
    const int64_t entries = int64_t(D.B) * D.Hkv * P.gl_total;
    float *dkc = nullptr, *dvc = nullptr;
    if (compact) {
        dkc = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + P.off_dkc);
        dvc = dkc + align256(size_t(entries) * 128 * 4) / 4;
    }
    if (entries > 0)
        LRSA_TIMED_LAUNCH("k_bwd_dkv_reduce", st, k_bwd_dkv_reduce, dim3((unsigned)((entries + 7) / 8)), dim3(256), 0, st, D,
                          idx, part, (bf16_t*)dK, (bf16_t*)dV, accK, accV, dkc, dvc, P);
    if (entries > 0 && compact)
        LRSA_TIMED_LAUNCH("k_bwd_scatter_dkv", st, k_bwd_scatter_dkv, dim3((unsigned)((entries + 7) / 8)), dim3(256), 0, st, D,
                          idx, dkc, dvc, (bf16_t*)dK, (bf16_t*)dV, P.gl_total);
    return hipGetLastError();
}

}  // namespace lrsa
