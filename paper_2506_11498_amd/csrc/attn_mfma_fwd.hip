// LRSA attention forward on bf16 MFMA (gfx950), head_dim 128: Eq. 2-3 of the paper under the
// chunked mask, flash style (online softmax, only the log-sum-exp is kept for the backward).
//
// One workgroup (8 waves) owns 256 (head, query) rows: GH query heads of one KV group x 256/GH
// consecutive queries of one segment (the sink, or one chunk); a wave owns 32 queries of one head.  The keys those queries see form one
// stream: the gather list (sink, then the survivors of the compressed chunks) followed by the
// contiguous local window up to the query itself.  Stream entry j is visible to query t iff
// j <= ng + t - cs, so only the last tiles need a mask.  The stream is walked in tiles of 64
// keys; K and V rows of a tile are copied (gathered by position) asynchronously from global
// memory straight into a four-stage LDS ring, three tiles ahead, row-major and swizzled.
//
// Per tile and wave:  S^T = K Q^T  (keys x queries, so a lane owns one query column and the
// softmax statistics are per lane), P^T = exp2(S^T - m), O^T += V^T P^T with the accumulator
// registers of S^T reused directly as the B operand and V^T read from the row-major tile with
// transposing LDS reads.
#include "mfma_tiles.h"

namespace lrsa {

constexpr int FWD_BN = 64;     // keys per tile
constexpr int FWD_WAVES = 8;   // waves per workgroup (two per SIMD), 32 queries each
constexpr int FWD_THREADS = 64 * FWD_WAVES;

// bf16, head_dim 128, and a head's K/V rows within 2 GiB of its first row (the copies use 32-bit byte offsets)
bool mfma_supported(const Dims& D) {
    return D.dtype == 1 && D.d == 128 && int64_t(D.n) * D.ks[2] * 2 < (int64_t(1) << 31);
}
size_t attn_fwd_mfma_ws_bytes(const Dims& D) { return compact_kv_bytes(D); }

// Copies the K and V rows of every gather-list entry into the condensed cache: 16 lanes per row, 16 rows
// per workgroup.
__global__ __launch_bounds__(256) void k_compact_kv(Dims D, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
                                                    const int32_t* __restrict__ idx, bf16_t* __restrict__ Kc,
                                                    bf16_t* __restrict__ Vc, int gl) {
    const int j = blockIdx.x * 16 + (threadIdx.x >> 4), sub = threadIdx.x & 15;
    const int bh = blockIdx.y;
    if (j >= gl) return;
    const int b = bh / D.Hkv, h = bh % D.Hkv;
    const int pos = j < D.S ? j : idx[int64_t(bh) * D.Ns * D.K + (j - D.S)];
    const int64_t src = b * D.ks[0] + h * D.ks[1] + int64_t(pos) * D.ks[2] + sub * 8;
    const int64_t dst = (int64_t(bh) * gl + j) * 128 + sub * 8;
    *reinterpret_cast<uint4*>(Kc + dst) = *reinterpret_cast<const uint4*>(K + src);
    *reinterpret_cast<uint4*>(Vc + dst) = *reinterpret_cast<const uint4*>(V + src);
}

hipError_t launch_compact_kv(const Dims& D, const void* K, const void* V, const int32_t* idx, void* Kc, void* Vc,
                             hipStream_t st) {
    const int gl = gather_list_len(D);
    if (gl == 0) return hipSuccess;
    LRSA_TIMED_LAUNCH("k_compact_kv", st, k_compact_kv, dim3((gl + 15) / 16, D.B * D.Hkv), dim3(256), 0, st, D,
                      (const bf16_t*)K, (const bf16_t*)V, idx, (bf16_t*)Kc, (bf16_t*)Vc, gl);
    return hipGetLastError();
}

// One 64-key tile of the walk for one wave: S^T = K Q^T, masked online softmax, O^T += V^T P^T.
struct FwdState {
    float m_run, l_run;
    f32x16 o[4];
};

// MASK: the tile holds entries some query of the wave does not see (only the last tiles of a walk).
// The running maximum is refreshed lazily: as long as no query's tile maximum exceeds its reference
// by more than 2^8, the old reference is kept (probabilities stay below 256, exact enough in fp32 sums
// and bf16 operands) and the accumulators need no rescaling.
template <bool MASK>
__device__ __forceinline__ void fwd_tile(const unsigned char* sK, const unsigned char* sV, const bf16x8 (&qf)[8],
                                         const LaneOffs& lo, FwdState& st, int j0, int lim, int wave_lim_max,
                                         float c2, int lane) {
    const int g = lane >> 5;
    // MASK tiles: do the second 32 keys hold a visible key for some query of the wave?
    const bool two = !MASK || j0 + 32 <= wave_lim_max;
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[kb][i] = 0.0f;
    // S^T = K Q^T: operands are read a block of 8 ahead of the MFMAs that consume them
    {
        bf16x8 a[8];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) a[kk] = read_rows_o(sK, lo, 0, kk);
        if (two) {
            bf16x8 a1[8];
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                s[0] = mfma32(a[kk], qf[kk], s[0]);
                a1[kk] = read_rows_o(sK, lo, 32, kk);
            }
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) s[1] = mfma32(a1[kk], qf[kk], s[1]);
            // keep the order written above -- 8 operand reads, then one read per MFMA, then 8 MFMAs: left alone,
            // the compiler moves every read down to just before its MFMA to save registers, and the MFMA then
            // waits out the whole LDS latency (0x100: LDS reads, 0x008: MFMAs)
            __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
        } else {
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) s[0] = mfma32(a[kk], qf[kk], s[0]);
        }
    }
    // first V^T operands are fetched while the softmax runs
    bf16x8 va[4], vb[4];
#pragma unroll
    for (int db = 0; db < 4; ++db) va[db] = read_cols_o(sV, lo, 0, db);
    float mx = -INFINITY;   // raw (unscaled) tile maximum of this lane's query
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (MASK) {
                const int j = j0 + kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
                s[kb][i] = j <= lim ? s[kb][i] : -INFINITY;
            }
            mx = fmaxf(mx, s[kb][i]);
        }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * c2;
    if (__builtin_amdgcn_ballot_w64(mx > st.m_run + 8.0f) != 0) {   // wave-uniform; always taken on the first tile
        const float m_new = fmaxf(st.m_run, mx);   // finite: the first tile holds a visible key for every query
        const float corr = fast_exp2(st.m_run - m_new);
        st.l_run *= corr;
        st.m_run = m_new;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) st.o[db][i] *= corr;
    }
    const float neg_m = -st.m_run;
    float psum = 0.0f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float pv = fast_exp2(__builtin_fmaf(s[kb][i], c2, neg_m));
            s[kb][i] = pv;
            psum += pv;
        }
    st.l_run += psum;
    // O^T += V^T P^T, 16 keys at a time; the operands of the next 16 keys are read during the MFMAs
#define LRSA_PV(kg, cur, nxt)                                                          \
    {                                                                                  \
        const bf16x8 pf = pack8(s[(kg) >> 1], 8 * ((kg) & 1));                         \
        _Pragma("unroll") for (int db = 0; db < 4; ++db) {                             \
            st.o[db] = mfma32(cur[db], pf, st.o[db]);                                  \
            if ((kg) + 1 < 4) nxt[db] = read_cols_o(sV, lo, ((kg) + 1) * 16, db);      \
        }                                                                              \
    }
    LRSA_PV(0, va, vb);
    LRSA_PV(1, vb, va);
    if (two) {
        LRSA_PV(2, va, vb);
        LRSA_PV(3, vb, va);
    }
#undef LRSA_PV
}

// GH query heads of one KV group share the workgroup: its 8 waves cover GH heads x QT = 256/GH queries,
// so every K/V tile staged in LDS serves 256 (head, query) rows.
// COMPACT: the rows of the gather list come from the condensed cache Kc, Vc (contiguous), no index is read.
template <int GH, bool COMPACT>
__global__ __launch_bounds__(FWD_THREADS, 2) void k_fwd_mfma(Dims D, const bf16_t* __restrict__ Q,
                                                              const bf16_t* __restrict__ K,
                                                              const bf16_t* __restrict__ V,
                                                              const int32_t* __restrict__ idx,
                                                              const bf16_t* __restrict__ Kc,
                                                              const bf16_t* __restrict__ Vc,
                                                              bf16_t* __restrict__ O, float* __restrict__ lse,
                                                              QTileMap M) {
    constexpr int WPH = FWD_WAVES / GH;   // waves per head
    constexpr int QT = 32 * WPH;          // queries per head and workgroup
    // four stages, each one array holding the K tile then the V tile; separate arrays per stage so that
    // reads of one stage need not wait for the asynchronous fill of another (the compiler tracks only a
    // handful of such arrays, hence K and V share one)
    constexpr int TILE_BYTES = FWD_BN * TILE_ROW_BYTES;
    __shared__ __attribute__((aligned(16))) unsigned char sT0[2 * TILE_BYTES], sT1[2 * TILE_BYTES], sT2[2 * TILE_BYTES],
        sT3[2 * TILE_BYTES];

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
    if (t0 >= seg_end) return;  // uniform for the workgroup
    const int t_last = min(t0 + QT, seg_end) - 1;
    const int ng = gather_count(D, qc), cs = window_start(D, qc);
    const int m_max = ng + t_last - cs + 1;           // stream entries the last row sees
    const int ntiles = (m_max + FWD_BN - 1) / FWD_BN;

    const bf16_t* Kh = K + b * D.ks[0] + h * D.ks[1];
    const bf16_t* Vh = V + b * D.ks[0] + h * D.ks[1];
    const int32_t* idx_h = idx + (int64_t(b) * D.Hkv + h) * D.Ns * D.K;
    const int64_t coff = COMPACT ? (int64_t(b) * D.Hkv + h) * (int64_t(D.S) + int64_t(D.K) * D.Ns) * 128 : 0;
    const bf16_t* Kc_h = Kc + coff;
    const bf16_t* Vc_h = Vc + coff;

    // this lane's query column
    const int tq = t0 + wq * 32 + l32;
    const int tq_ld = tq < t_last ? tq : t_last;
    bf16x8 qf[8];
    {
        const bf16_t* qrow = Q + b * D.qs[0] + hq * D.qs[1] + int64_t(tq_ld) * D.qs[2];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qrow + kk * 16 + g * 8);
    }
    const int lim = ng + tq - cs;                                     // last stream entry this query sees
    const int wave_lim_max = ng + min(t0 + wq * 32 + 31, t_last) - cs;  // ... the wave's last valid query sees
    const int wave_lim_min = ng + t0 + wq * 32 - cs;                    // ... the wave's first query sees

    // loader: wave w fills tile rows 8w .. 8w+7 with two asynchronous copies of 4 rows each (K and V:
    // 4 copies per tile); rows past the stream end re-read its last key and are masked.  The 8 stream
    // positions a wave needs per tile are wave-uniform addresses, so they are fetched through the scalar
    // cache (one iteration ahead); the only vector memory operations in the loop are the asynchronous
    // copies, always 4 per wave and tile, which lets s_waitcnt vmcnt(n) address a tile.
    const int32_t* idx_ld = D.Ns > 0 ? idx_h : reinterpret_cast<const int32_t*>(Kh);   // any readable words
    const int idx_last = D.Ns > 0 ? D.Ns * D.K - 1 : 0;
    const int wv = __builtin_amdgcn_readfirstlane(wave);
    auto pos_entry = [&](int tc, int r) {   // clamped index into idx of row r of the wave's 8 tile rows
        const int e = min(tc * FWD_BN + 8 * wv + r, m_max - 1) - D.S;
        return e < 0 ? 0 : (e > idx_last ? idx_last : e);
    };
    auto fetch_pos = [&](int tile, Scalar8& raw) {
        if (COMPACT) return;
        const int tc = tile < ntiles ? tile : ntiles - 1;   // past the end: repeat the last tile (never consumed)
        raw.a0 = smem_load(idx_ld, pos_entry(tc, 0)); raw.a1 = smem_load(idx_ld, pos_entry(tc, 1));
        raw.a2 = smem_load(idx_ld, pos_entry(tc, 2)); raw.a3 = smem_load(idx_ld, pos_entry(tc, 3));
        raw.a4 = smem_load(idx_ld, pos_entry(tc, 4)); raw.a5 = smem_load(idx_ld, pos_entry(tc, 5));
        raw.a6 = smem_load(idx_ld, pos_entry(tc, 6)); raw.a7 = smem_load(idx_ld, pos_entry(tc, 7));
    };
    // laK, laV: LDS byte addresses of the stage's K tile and V tile (compile-time constants at the call sites)
    auto issue = [&](int tile, Scalar8& raw, unsigned laK, unsigned laV) {
        const int tc = tile < ntiles ? tile : ntiles - 1;
        const int q4 = lane >> 4;
        if (!COMPACT) smem_wait(raw);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r4 = 8 * wv + 4 * i;
            int j = tc * FWD_BN + r4 + q4;
            j = j < m_max ? j : m_max - 1;
            const int ch = async_chunk(r4 + q4, lane) * 8;
            const unsigned row_la = unsigned(r4) * TILE_ROW_BYTES;      // wave-uniform
            if (COMPACT) {
                async_copy16_la(stream_row(Kc_h, Kh, D.ks[2], j, ng, cs) + ch, laK + row_la);
                async_copy16_la(stream_row(Vc_h, Vh, D.ks[2], j, ng, cs) + ch, laV + row_la);
            } else {
                const int sel = i == 0 ? pick4(q4, raw.a0, raw.a1, raw.a2, raw.a3) : pick4(q4, raw.a4, raw.a5, raw.a6, raw.a7);
                const int pos = j < ng ? (j < D.S ? j : sel) : cs + (j - ng);
                // byte offset inside the head: below 2^31 (a condition of this kernel, checked on the host)
                const unsigned off = (unsigned(pos) * unsigned(D.ks[2]) + unsigned(ch)) * 2u;
                async_copy16_so(Kh, off, laK + row_la);
                async_copy16_so(Vh, off, laV + row_la);
            }
        }
    };
    constexpr int OPS_PER_TILE = 4;   // asynchronous copies per wave and tile

    const float c2 = D.scale * 1.4426950408889634f;  // logits are kept in log2 units
    const LaneOffs lo = make_lane_offs(lane);
    FwdState st;
    st.m_run = -INFINITY;
    st.l_run = 0.0f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) st.o[db][i] = 0.0f;

#define LRSA_FWD_TILE(sK, sV, j0_)                                                                   \
    {                                                                                                \
        const int j0 = (j0_);                                                                        \
        if (j0 + FWD_BN - 1 <= wave_lim_min) fwd_tile<false>(sK, sV, qf, lo, st, j0, lim, wave_lim_max, c2, lane); \
        else if (j0 <= wave_lim_max) fwd_tile<true>(sK, sV, qf, lo, st, j0, lim, wave_lim_max, c2, lane);          \
    }

    // A wave's vector memory operations in order:  A(0) A(1) A(2) | iteration t: A(t+3)   (A = the copies
    // of a tile).  At the top of iteration t the operations issued after A(t) are A(t+1) A(t+2).
    Scalar8 posA, posB;
    const unsigned la0 = lds_addr(sT0), la1 = lds_addr(sT1), la2 = lds_addr(sT2), la3 = lds_addr(sT3);
    fetch_pos(0, posA); issue(0, posA, la0, la0 + TILE_BYTES);
    fetch_pos(1, posB); issue(1, posB, la1, la1 + TILE_BYTES);
    fetch_pos(2, posA); issue(2, posA, la2, la2 + TILE_BYTES);
    fetch_pos(3, posB);
    wait_all_vmem_known();   // the Q fragments (and the first tiles) are here
#define LRSA_FWD_STEP(t_, sT, laN, pos_use, pos_fetch)                                               \
    {                                                                                                \
        wait_vmcnt<2 * OPS_PER_TILE>();   /* this wave's copies for tile t_ have landed */            \
        ring_barrier();                   /* everybody's have; everybody is done with tile t_-1 */   \
        issue((t_) + 3, pos_use, laN, laN + TILE_BYTES); /* tile t_+3 into the stage tile t_-1 used */ \
        fetch_pos((t_) + 4, pos_fetch);   /* after the copies: their wait for positions is for ALL scalar loads */ \
        LRSA_FWD_TILE(sT, sT + TILE_BYTES, (t_) * FWD_BN);                                           \
    }
    for (int tile = 0; tile < ntiles; tile += 4) {
        LRSA_FWD_STEP(tile, sT0, la3, posB, posA);
        if (tile + 1 >= ntiles) break;
        LRSA_FWD_STEP(tile + 1, sT1, la0, posA, posB);
        if (tile + 2 >= ntiles) break;
        LRSA_FWD_STEP(tile + 2, sT2, la1, posB, posA);
        if (tile + 3 >= ntiles) break;
        LRSA_FWD_STEP(tile + 3, sT3, la2, posA, posB);
    }
#undef LRSA_FWD_STEP
    wait_vmcnt<0>();   // copies issued past the end must land before the workgroup's LDS is released
#undef LRSA_FWD_TILE

    const float l_tot = st.l_run + __shfl_xor(st.l_run, 32, 64);
    if (tq <= t_last) {
        const float inv = 1.0f / l_tot;
        bf16_t* orow = O + b * D.qs[0] + hq * D.qs[1] + int64_t(tq) * D.qs[2];
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                f32x4 v;
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = st.o[db][a * 4 + r] * inv;
                const bf16x4 pk = __builtin_convertvector(v, bf16x4);
                *reinterpret_cast<bf16x4*>(orow + db * 32 + a * 8 + g * 4) = pk;
            }
        if (g == 0) lse[(int64_t(b) * D.Hq + hq) * D.lse_stride + tq] = (st.m_run + __builtin_log2f(l_tot)) * 0.6931471805599453f;
    }
}

hipError_t launch_attn_fwd_mfma(const Dims& D, const void* Q, const void* K, const void* V, const int32_t* idx,
                                void* O, float* lse, void* ws, hipStream_t st) {
    const int gh = heads_per_wg(D);
    const QTileMap M = make_qtile_map(D, gh, FWD_WAVES);
    const int64_t wgs = int64_t(D.B) * D.Hkv * M.per_unit;
    if (wgs == 0) return hipSuccess;
    const bf16_t *q = (const bf16_t*)Q, *k = (const bf16_t*)K, *v = (const bf16_t*)V;
    const bool compact = D.compact && gather_list_len(D) > 0;
    const bf16_t *kc = nullptr, *vc = nullptr;
    if (compact) {
        kc = reinterpret_cast<const bf16_t*>(ws);
        vc = reinterpret_cast<const bf16_t*>(reinterpret_cast<const char*>(ws) + compact_kv_bytes(D) / 2);
        const hipError_t e = launch_compact_kv(D, K, V, idx, (void*)kc, (void*)vc, st);
        if (e != hipSuccess) return e;
    }
#define LRSA_FWD_LAUNCH(GH_, C_)                                                                                   \
    LRSA_TIMED_LAUNCH("k_fwd_mfma", st, (k_fwd_mfma<GH_, C_>), dim3((unsigned)wgs), dim3(FWD_THREADS), 0, st, D, q, k, v, \
                      idx, kc, vc, (bf16_t*)O, lse, M)
    if (gh == 4) { if (compact) LRSA_FWD_LAUNCH(4, true); else LRSA_FWD_LAUNCH(4, false); }
    else if (gh == 2) { if (compact) LRSA_FWD_LAUNCH(2, true); else LRSA_FWD_LAUNCH(2, false); }
    else { if (compact) LRSA_FWD_LAUNCH(1, true); else LRSA_FWD_LAUNCH(1, false); }
#undef LRSA_FWD_LAUNCH
    return hipGetLastError();
}

}  // namespace lrsa
