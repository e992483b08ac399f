// LRSA attention backward on bf16 MFMA (gfx950), head_dim 128.  Gradients of sum(O * dO) with
// the mask constant:  A = exp(scale Q K^T + M - lse), dV = A^T dO, dA = dO V^T,
// D = rowsum(dO * O), dS = A * (dA - D), dQ = scale dS K, dK = scale dS^T Q.
//
// Deterministic, no atomics.  Four launches on one stream:
//   k_bwd_rowdot   D[b,hq,t] = dO[t] . O[t]
//   k_bwd_dq       query-outer: a workgroup owns 128 queries and walks their key stream exactly
//                  like the forward (gather list, then the local window), recomputing A
//   k_bwd_dkv      key-outer, mode GATHER: a workgroup owns 128 consecutive entries of one KV
//                  head's gather list (sink ++ survivors) and a range of query chunks; it writes
//                  fp32 partial dK, dV rows for those entries into the workspace
//   k_bwd_dkv      key-outer, mode WINDOW: a workgroup owns 128 consecutive positions and walks
//                  the queries that see them through the local window (own chunk causally, the
//                  next local_prev chunks in full); its epilogue adds the GATHER partials of the
//                  positions that are sink tokens or survivors, scales and writes dK, dV.
// In the key-outer kernel a lane owns one key column of S = Q K^T, so K and V fragments stay in
// registers for the whole walk; Q and dO rows stream through LDS 32 rows at a time and are read
// both row-wise (for S and dA) and transposed (for dV^T += dO^T A and dK^T += Q^T dS).
#include "mfma_tiles.h"

namespace lrsa {

constexpr int BWD_THREADS = 256;
constexpr int DQ_BM = 128, DQ_BN = 64;
constexpr int KV_BK = 128;  // keys per workgroup (32 per wave)
constexpr int KV_BQ = 32;   // query rows per step
constexpr int KV_MAX_SLICES = 8;

// ------------------------------------------------------------------------------------ host-side plan
struct BwdPlan {
    int sink_tiles_q, tpc_q;    // dQ: query tiles of 128
    int sink_tiles_k, tpc_k;    // dK/dV window mode: key tiles of 128
    int gl_total, gtiles;       // gather list length per KV head, its tiles of 128
    int qch, nsl;               // query chunks per slice, slices per gather tile (<= KV_MAX_SLICES)
    size_t off_part, bytes;     // workspace: D first, then the fp32 partials
};

static BwdPlan make_plan(const Dims& D) {
    BwdPlan P;
    const int sink_rows = D.S < D.n ? D.S : D.n;
    P.sink_tiles_q = (sink_rows + DQ_BM - 1) / DQ_BM;
    P.tpc_q = (D.L + DQ_BM - 1) / DQ_BM;
    P.sink_tiles_k = (sink_rows + KV_BK - 1) / KV_BK;
    P.tpc_k = (D.L + KV_BK - 1) / KV_BK;
    P.gl_total = D.nq > 0 ? D.S + D.K * D.Ns : 0;
    P.gtiles = (P.gl_total + KV_BK - 1) / KV_BK;
    // aim at ~512 steps of 32 rows per workgroup, but never more than KV_MAX_SLICES slices
    int64_t qch = (512 * int64_t(KV_BQ)) / (int64_t(D.L) * D.G);
    if (qch < 1) qch = 1;
    const int min_qch = (D.nq + KV_MAX_SLICES - 1) / KV_MAX_SLICES;
    if (qch < min_qch) qch = min_qch;
    if (qch < 1) qch = 1;
    P.qch = int(qch);
    P.nsl = D.nq > 0 ? (D.nq + P.qch - 1) / P.qch : 0;
    P.off_part = align256(size_t(D.B) * D.Hq * D.n * 4);
    const size_t part = size_t(2) * P.nsl * D.B * D.Hkv * P.gl_total * 128 * 4;
    P.bytes = P.off_part + align256(part);
    return P;
}

size_t attn_bwd_mfma_ws_bytes(const Dims& D) { return make_plan(D).bytes; }

// ------------------------------------------------------------------------------------ D = rowsum(dO * O)
__global__ __launch_bounds__(BWD_THREADS) void k_bwd_rowdot(Dims D, const bf16_t* __restrict__ O,
                                                             const bf16_t* __restrict__ dO,
                                                             float* __restrict__ Dsum) {
    // 16 lanes per row, 16 rows per workgroup
    const int sub = threadIdx.x & 15;
    const int64_t row = int64_t(blockIdx.x) * 16 + (threadIdx.x >> 4);
    const int64_t nrows = int64_t(D.B) * D.Hq * D.n;
    float acc = 0.0f;
    if (row < nrows) {
        const int t = int(row % D.n);
        const int hq = int((row / D.n) % D.Hq), b = int(row / (int64_t(D.n) * D.Hq));
        const int64_t off = b * D.qs[0] + hq * D.qs[1] + int64_t(t) * D.qs[2] + sub * 8;
        float a[8], c[8];
        Elem<bf16_t>::load(O + off, a);
        Elem<bf16_t>::load(dO + off, c);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc += a[i] * c[i];
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (row < nrows && sub == 0) Dsum[row] = acc;
}

// ------------------------------------------------------------------------------------ dQ
__global__ __launch_bounds__(BWD_THREADS, 2) void k_bwd_dq(Dims D, const bf16_t* __restrict__ Q,
                                                            const bf16_t* __restrict__ K,
                                                            const bf16_t* __restrict__ V,
                                                            const bf16_t* __restrict__ dO,
                                                            const float* __restrict__ lse,
                                                            const float* __restrict__ Dsum,
                                                            const int32_t* __restrict__ idx,
                                                            bf16_t* __restrict__ dQ, int sink_tiles, int tpc) {
    __shared__ __attribute__((aligned(16))) unsigned char sK[DQ_BN * TILE_ROW_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char sV[DQ_BN * TILE_ROW_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int hq = blockIdx.y, b = blockIdx.z, h = hq / D.G;

    const int tix = gridDim.x - 1 - blockIdx.x;
    int qc, t0, seg_end;
    if (tix < sink_tiles) {
        qc = -1; t0 = tix * DQ_BM; seg_end = D.S < D.n ? D.S : D.n;
    } else {
        const int tt = tix - sink_tiles;
        qc = tt / tpc;
        t0 = D.S + qc * D.L + (tt % tpc) * DQ_BM;
        const int64_t e = int64_t(D.S) + int64_t(qc + 1) * D.L;
        seg_end = e < D.n ? int(e) : D.n;
    }
    if (t0 >= seg_end) return;
    const int t_last = min(t0 + DQ_BM, seg_end) - 1;
    const int ng = gather_count(D, qc), cs = window_start(D, qc);
    const int m_max = ng + t_last - cs + 1;
    const int ntiles = (m_max + DQ_BN - 1) / DQ_BN;

    const bf16_t* Kh = K + b * D.ks[0] + h * D.ks[1];
    const bf16_t* Vh = V + b * D.ks[0] + h * D.ks[1];
    const int32_t* idx_h = idx + (int64_t(b) * D.Hkv + h) * D.Ns * D.K;

    const int tq = t0 + wave * 32 + l32;
    const int tq_ld = tq < t_last ? tq : t_last;
    const int64_t qoff = b * D.qs[0] + hq * D.qs[1] + int64_t(tq_ld) * D.qs[2];
    bf16x8 qf[8], gf[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        qf[kk] = *reinterpret_cast<const bf16x8*>(Q + qoff + kk * 16 + g * 8);
        gf[kk] = *reinterpret_cast<const bf16x8*>(dO + qoff + kk * 16 + g * 8);
    }
    const int64_t rowid = (int64_t(b) * D.Hq + hq) * D.n + tq_ld;
    const float lse2 = lse[rowid] * 1.4426950408889634f;
    const float Dq = Dsum[rowid];
    const int lim = ng + tq - cs;
    const int wave_lim_max = ng + min(t0 + wave * 32 + 31, t_last) - cs;

    const int kg4 = tid >> 4, c16 = tid & 15;
    int pos0, pos1, pos2, pos3;
    uint4 kr0, kr1, kr2, kr3, vr0, vr1, vr2, vr3;
#define LRSA_POS(tile, e) stream_pos(D, idx_h, min((tile) * DQ_BN + 4 * kg4 + (e), m_max - 1), ng, cs)
#define LRSA_FETCH_POS(tile) { pos0 = LRSA_POS(tile, 0); pos1 = LRSA_POS(tile, 1); pos2 = LRSA_POS(tile, 2); pos3 = LRSA_POS(tile, 3); }
#define LRSA_LD(base, p) (*reinterpret_cast<const uint4*>((base) + int64_t(p) * D.ks[2] + c16 * 8))
#define LRSA_ISSUE() { kr0 = LRSA_LD(Kh, pos0); kr1 = LRSA_LD(Kh, pos1); kr2 = LRSA_LD(Kh, pos2); kr3 = LRSA_LD(Kh, pos3); \
                       vr0 = LRSA_LD(Vh, pos0); vr1 = LRSA_LD(Vh, pos1); vr2 = LRSA_LD(Vh, pos2); vr3 = LRSA_LD(Vh, pos3); }
#define LRSA_ST(tile_base, e, v) (*reinterpret_cast<uint4*>((tile_base) + tile_off(4 * kg4 + (e), c16)) = (v))
#define LRSA_STASH() { LRSA_ST(sK, 0, kr0); LRSA_ST(sK, 1, kr1); LRSA_ST(sK, 2, kr2); LRSA_ST(sK, 3, kr3); \
                       LRSA_ST(sV, 0, vr0); LRSA_ST(sV, 1, vr1); LRSA_ST(sV, 2, vr2); LRSA_ST(sV, 3, vr3); }

    const float c2 = D.scale * 1.4426950408889634f;
    f32x16 dq[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dq[db][i] = 0.0f;

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
        const int j0 = tile * DQ_BN;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            if (j0 + kb * 32 <= wave_lim_max) {  // otherwise these 32 keys are masked for the whole wave
                f32x16 s, dp;
#pragma unroll
                for (int i = 0; i < 16; ++i) { s[i] = 0.0f; dp[i] = 0.0f; }
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) s = mfma32(read_rows(sK, kb * 32, kk, l32, g), qf[kk], s);
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) dp = mfma32(read_rows(sV, kb * 32, kk, l32, g), gf[kk], dp);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int j = j0 + kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
                    const float pr = j <= lim ? fast_exp2(s[i] * c2 - lse2) : 0.0f;
                    s[i] = pr * (dp[i] - Dq);
                }
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    const bf16x8 dsf = pack8(s, 8 * hh);
#pragma unroll
                    for (int db = 0; db < 4; ++db)
                        dq[db] = mfma32(read_cols(sK, kb * 32 + hh * 16, db, lane), dsf, dq[db]);
                }
            }
        }
        __syncthreads();
    }
#undef LRSA_POS
#undef LRSA_FETCH_POS
#undef LRSA_LD
#undef LRSA_ISSUE
#undef LRSA_ST
#undef LRSA_STASH

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

template <bool GATHER>
__global__ __launch_bounds__(BWD_THREADS, 2) void k_bwd_dkv(Dims D, const bf16_t* __restrict__ Q,
                                                             const bf16_t* __restrict__ K,
                                                             const bf16_t* __restrict__ V,
                                                             const bf16_t* __restrict__ dO,
                                                             const float* __restrict__ lse,
                                                             const float* __restrict__ Dsum,
                                                             const int32_t* __restrict__ idx,
                                                             bf16_t* __restrict__ dK, bf16_t* __restrict__ dV,
                                                             float* __restrict__ part, BwdPlan P) {
    __shared__ __attribute__((aligned(16))) unsigned char sQ[KV_BQ * TILE_ROW_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char sG[KV_BQ * TILE_ROW_BYTES];
    __shared__ __attribute__((aligned(16))) float sL[KV_BQ];   // lse in log2 units
    __shared__ __attribute__((aligned(16))) float sD[KV_BQ];   // D
    __shared__ __attribute__((aligned(16))) int sLim[KV_BQ];   // largest key id the row sees (-1: none)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int h = blockIdx.y, b = blockIdx.z;
    const int32_t* idx_h = idx + (int64_t(b) * D.Hkv + h) * D.Ns * D.K;

    // ---- which keys, which query rows
    int key0, key_end;   // key ids of this workgroup: positions (WINDOW) or gather-list entries (GATHER)
    int ta, tb;          // query rows [ta, tb) of every head of the group
    int slice = 0;
    if (GATHER) {
        const int jt = blockIdx.x / P.nsl;
        slice = blockIdx.x % P.nsl;
        key0 = jt * KV_BK;
        key_end = P.gl_total;
        const int qa = first_chunk_seeing(D, key0) + slice * P.qch;
        if (qa >= D.nq) return;
        const int qb = min(D.nq, qa + P.qch);
        ta = D.S + qa * D.L;
        const int64_t e = int64_t(D.S) + int64_t(qb) * D.L;
        tb = e < D.n ? int(e) : D.n;
    } else {
        const int tix = gridDim.x - 1 - blockIdx.x;
        if (tix < P.sink_tiles_k) {
            key0 = tix * KV_BK;
            key_end = D.S < D.n ? D.S : D.n;
            tb = key_end;                         // only sink queries see sink keys through the window
        } else {
            const int tt = tix - P.sink_tiles_k;
            const int kc = tt / P.tpc_k;
            key0 = D.S + kc * D.L + (tt % P.tpc_k) * KV_BK;
            const int64_t e = int64_t(D.S) + int64_t(kc + 1) * D.L;
            key_end = e < D.n ? int(e) : D.n;
            const int64_t e2 = int64_t(D.S) + (int64_t(kc) + 1 + D.lp) * D.L;
            tb = e2 < D.n ? int(e2) : D.n;
        }
        if (key0 >= key_end) return;
        ta = key0;
    }
    const int nr = tb - ta;
    const int sph = (nr + KV_BQ - 1) / KV_BQ;   // steps per head
    const int nsteps = sph * D.G;

    // ---- this lane's key column: fragments of K and V stay in registers
    const int kid = key0 + wave * 32 + l32;
    const bool kvalid = kid < key_end;
    const int kid_ld = kvalid ? kid : key_end - 1;
    const int kpos = GATHER ? (kid_ld < D.S ? kid_ld : idx_h[kid_ld - D.S]) : kid_ld;
    const int kcmp = kvalid ? kid : 0x7fffffff;
    bf16x8 kf[8], vf[8];
    {
        const int64_t koff = b * D.ks[0] + h * D.ks[1] + int64_t(kpos) * D.ks[2];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            kf[kk] = *reinterpret_cast<const bf16x8*>(K + koff + kk * 16 + g * 8);
            vf[kk] = *reinterpret_cast<const bf16x8*>(V + koff + kk * 16 + g * 8);
        }
    }
    const int wave_key0 = key0 + wave * 32;

    // ---- loader: thread takes row tid/8 of the step, chunks 2*(tid%8) and +1 of Q and dO
    const int lrow = tid >> 3, lc = (tid & 7) * 2;
    uint4 q0, q1, g0, g1;
    float r_l = 0.0f, r_d = 0.0f;
    int r_lim = -1;
#define LRSA_ISSUE(step)                                                                              \
    {                                                                                                 \
        const int gi_ = (step) / sph, r0_ = ta + ((step) % sph) * KV_BQ;                              \
        const int t_ = min(r0_ + lrow, tb - 1);                                                       \
        const int hq_ = h * D.G + gi_;                                                                \
        const int64_t off_ = b * D.qs[0] + hq_ * D.qs[1] + int64_t(t_) * D.qs[2] + lc * 8;             \
        q0 = *reinterpret_cast<const uint4*>(Q + off_);                                               \
        q1 = *reinterpret_cast<const uint4*>(Q + off_ + 8);                                           \
        g0 = *reinterpret_cast<const uint4*>(dO + off_);                                              \
        g1 = *reinterpret_cast<const uint4*>(dO + off_ + 8);                                          \
        if (tid < KV_BQ) {                                                                            \
            const int tt_ = r0_ + tid;                                                                \
            const int tc_ = min(tt_, tb - 1);                                                         \
            const int64_t rid_ = (int64_t(b) * D.Hq + hq_) * D.n + tc_;                               \
            r_l = lse[rid_] * 1.4426950408889634f;                                                    \
            r_d = Dsum[rid_];                                                                         \
            if (tt_ >= tb) r_lim = -1;                                                                \
            else if (GATHER) r_lim = gather_count(D, (tt_ - D.S) / D.L) - 1;                          \
            else r_lim = tt_;                                                                         \
        }                                                                                             \
    }
#define LRSA_STASH()                                                                                  \
    {                                                                                                 \
        *reinterpret_cast<uint4*>(sQ + tile_off(lrow, lc)) = q0;                                      \
        *reinterpret_cast<uint4*>(sQ + tile_off(lrow, lc + 1)) = q1;                                  \
        *reinterpret_cast<uint4*>(sG + tile_off(lrow, lc)) = g0;                                      \
        *reinterpret_cast<uint4*>(sG + tile_off(lrow, lc + 1)) = g1;                                  \
        if (tid < KV_BQ) { sL[tid] = r_l; sD[tid] = r_d; sLim[tid] = r_lim; }                         \
    }

    const float c2 = D.scale * 1.4426950408889634f;
    f32x16 dk[4], dv[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) { dk[db][i] = 0.0f; dv[db][i] = 0.0f; }

    LRSA_ISSUE(0);
    for (int step = 0; step < nsteps; ++step) {
        LRSA_STASH();
        __syncthreads();
        if (step + 1 < nsteps) LRSA_ISSUE(step + 1);
        const int r0 = ta + (step % sph) * KV_BQ;
        // WINDOW: rows before the wave's first key see none of its keys
        if (GATHER || r0 + KV_BQ - 1 >= wave_key0) {
            f32x16 s, dp;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s[i] = 0.0f; dp[i] = 0.0f; }
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) s = mfma32(read_rows(sQ, 0, kk, l32, g), kf[kk], s);
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) dp = mfma32(read_rows(sG, 0, kk, l32, g), vf[kk], dp);
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int rb = 8 * a + 4 * g;
                const f32x4 l4 = *reinterpret_cast<const f32x4*>(sL + rb);
                const f32x4 d4 = *reinterpret_cast<const f32x4*>(sD + rb);
                const int4 m4 = *reinterpret_cast<const int4*>(sLim + rb);
                const int lims[4] = {m4.x, m4.y, m4.z, m4.w};
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int i = a * 4 + r;
                    const float pr = kcmp <= lims[r] ? fast_exp2(s[i] * c2 - l4[r]) : 0.0f;
                    s[i] = pr;
                    dp[i] = pr * (dp[i] - d4[r]);
                }
            }
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const bf16x8 pf = pack8(s, 8 * hh);
                const bf16x8 dsf = pack8(dp, 8 * hh);
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    dv[db] = mfma32(read_cols(sG, hh * 16, db, lane), pf, dv[db]);
                    dk[db] = mfma32(read_cols(sQ, hh * 16, db, lane), dsf, dk[db]);
                }
            }
        }
        __syncthreads();
    }
#undef LRSA_ISSUE
#undef LRSA_STASH

    if (!kvalid) return;
    const size_t part_stride = size_t(D.B) * D.Hkv * P.gl_total * 128;   // floats per slice
    const size_t part_v = size_t(P.nsl) * part_stride;                    // dV partials follow the dK partials
    if (GATHER) {
        float* pk = part + size_t(slice) * part_stride + ((size_t(b) * D.Hkv + h) * P.gl_total + kid) * 128;
        float* pv = pk + part_v;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                f32x4 x, y;
#pragma unroll
                for (int r = 0; r < 4; ++r) { x[r] = dk[db][a * 4 + r] * D.scale; y[r] = dv[db][a * 4 + r]; }
                *reinterpret_cast<f32x4*>(pk + db * 32 + a * 8 + g * 4) = x;
                *reinterpret_cast<f32x4*>(pv + db * 32 + a * 8 + g * 4) = y;
            }
    } else {
        // gather-list entry of this position, if it is a sink token or a survivor
        int j = -1;
        if (P.gtiles > 0) {
            if (kid < D.S) j = kid;
            else {
                const int c = (kid - D.S) / D.L;
                if (c < D.Ns) {
                    const int32_t* rowp = idx_h + int64_t(c) * D.K;
                    int lo = 0, hi = D.K - 1;
                    while (lo <= hi) {
                        const int mid = (lo + hi) >> 1;
                        const int v = rowp[mid];
                        if (v == kid) { j = D.S + c * D.K + mid; break; }
                        if (v < kid) lo = mid + 1; else hi = mid - 1;
                    }
                }
            }
        }
        int nrng = 0;
        const float* pk = nullptr;
        if (j >= 0) {
            const int qf0 = first_chunk_seeing(D, (j / KV_BK) * KV_BK);
            nrng = qf0 < D.nq ? (D.nq - qf0 + P.qch - 1) / P.qch : 0;
            pk = part + ((size_t(b) * D.Hkv + h) * P.gl_total + j) * 128;
        }
        const int64_t koff = b * D.ks[0] + h * D.ks[1] + int64_t(kid) * D.ks[2];
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                f32x4 x, y;
#pragma unroll
                for (int r = 0; r < 4; ++r) { x[r] = dk[db][a * 4 + r] * D.scale; y[r] = dv[db][a * 4 + r]; }
                const int dcol = db * 32 + a * 8 + g * 4;
                for (int sidx = 0; sidx < nrng; ++sidx) {
                    x += *reinterpret_cast<const f32x4*>(pk + size_t(sidx) * part_stride + dcol);
                    y += *reinterpret_cast<const f32x4*>(pk + part_v + size_t(sidx) * part_stride + dcol);
                }
                *reinterpret_cast<bf16x4*>(dK + koff + dcol) = __builtin_convertvector(x, bf16x4);
                *reinterpret_cast<bf16x4*>(dV + koff + dcol) = __builtin_convertvector(y, bf16x4);
            }
    }
}

// ------------------------------------------------------------------------------------ launcher
hipError_t launch_attn_bwd_mfma(const Dims& D, const void* Q, const void* K, const void* V, const void* O,
                                const void* dO, const float* lse, const int32_t* idx, void* dQ, void* dK,
                                void* dV, void* ws, hipStream_t st) {
    const BwdPlan P = make_plan(D);
    float* Dsum = reinterpret_cast<float*>(ws);
    float* part = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + P.off_part);
    const bf16_t *q = (const bf16_t*)Q, *k = (const bf16_t*)K, *v = (const bf16_t*)V, *o = (const bf16_t*)O,
                 *g = (const bf16_t*)dO;

    const int64_t nrows = int64_t(D.B) * D.Hq * D.n;
    LRSA_TIMED_LAUNCH("k_bwd_rowdot", st, k_bwd_rowdot, dim3((unsigned)((nrows + 15) / 16)), dim3(BWD_THREADS), 0, st, D, o, g, Dsum);

    const int qtiles = P.sink_tiles_q + D.nq * P.tpc_q;
    if (qtiles > 0)
        LRSA_TIMED_LAUNCH("k_bwd_dq", st, k_bwd_dq, dim3(qtiles, D.Hq, D.B), dim3(BWD_THREADS), 0, st, D, q, k, v, g, lse, Dsum, idx,
                           (bf16_t*)dQ, P.sink_tiles_q, P.tpc_q);
    if (P.gtiles > 0)
        LRSA_TIMED_LAUNCH("k_bwd_dkvtrue", st, k_bwd_dkv<true>, dim3(P.gtiles * P.nsl, D.Hkv, D.B), dim3(BWD_THREADS), 0, st, D, q, k, v,
                           g, lse, Dsum, idx, (bf16_t*)dK, (bf16_t*)dV, part, P);
    const int ktiles = P.sink_tiles_k + D.nq * P.tpc_k;
    if (ktiles > 0)
        LRSA_TIMED_LAUNCH("k_bwd_dkvfalse", st, k_bwd_dkv<false>, dim3(ktiles, D.Hkv, D.B), dim3(BWD_THREADS), 0, st, D, q, k, v, g, lse,
                           Dsum, idx, (bf16_t*)dK, (bf16_t*)dV, part, P);
    return hipGetLastError();
}

}  // namespace lrsa
