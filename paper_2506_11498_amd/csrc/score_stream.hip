// Streaming LagKV scoring for bf16 data with head_dim 128 (Eq. 4-8 of the paper): every K and V row is read
// from memory ONCE.
//
// Eq. 6 normalises chunk p with the per-channel min / max of chunk p+1 (Eq. 4-5), so a walk over the chunks
// in DESCENDING order knows the reference statistics of a chunk before it meets the chunk: while the rows of
// chunk c stream through, their standard deviations (Eq. 7) are taken with the min / max of chunk c+1 and, in
// the same pass, the min / max of chunk c itself are collected for chunk c-1.
//
// A *stream* is one (batch, KV head, K or V) tensor.  Its chunks are cut into `ranges` (a range reads one extra
// chunk, the reference of its top chunk) and every chunk's rows into W row slices; one persistent workgroup
// owns (stream, range, slice) and walks its slice of every chunk of the range, top down.  The W sibling
// workgroups of a (stream, range) need each other's partial min / max of a chunk before they can score the
// chunk below it.  They exchange them through mailboxes in device memory that belongs to the library:
//   * a word is {tag : 32, max : bf16, min : bf16} of one channel, written and read as ONE 8-byte access;
//     the tag names the call and the chunk, so a reader knows whether the word it sees is the one it wants;
//   * a sibling publishes the 128 words of its slice and reads those of the other sibling (W <= 2: one memory
//     round trip, 1 KB per chunk against the >= 64 KB of rows a slice holds);
//   * the mailboxes are hints only: a reader that does not find its tag in time computes the min / max of
//     the reference chunk from the rows themselves.  Whatever the mailboxes hold, results are the same.
// To keep the exchange off the critical path the rows of a chunk stay in LDS for SS_LAG more blocks after
// their min / max have been taken and are scored only then; rows are copied from global memory straight into
// an LDS ring (asynchronous copies, SS_PF blocks ahead) by four of the sixteen waves, a fifth collects the
// siblings' words, a sixth publishes this workgroup's and writes the standard deviations out, all sixteen compute.
//
// A second kernel takes the softmax over each chunk's tokens for K and V, adds them (Eq. 7-8), optionally
// selects the top K (text after Eq. 8), and clears the mailboxes the call used.
//
// How the work is cut (host side): ranges first (a range of >= 8 chunks costs at most 1/8 more reads), then two
// slices per chunk, then shorter ranges; a slice holds at least two blocks of rows, so that at most one exchange
// is under way per workgroup.  The kernel is used when that cut fills three quarters of the CUs with at most 15 %
// of the rows read twice; other shapes go to the fused one-workgroup-per-chunk kernel (score.hip).
//
// Arithmetic: min / max are exact (packed 16-bit compares on the stored bf16 patterns); Eq. 6 is evaluated as
// z * (1 / den) - min / den, shifted by 1/2 so that the normalised values centre on zero; the variance over
// the channels is sum(x^2) - sum(x)^2 / d in fp32 and is recomputed from the deviations when the two terms
// cancel.  Values of magnitude >= 2^121 or NaN are outside the contract (their bf16 patterns do not order
// like numbers in a 16-bit float compare).
#include "mfma_tiles.h"
#include "score_block.h"
#include "select_block.h"

#include <atomic>
#include <mutex>

namespace lrsa {

constexpr int SS_THREADS = 1024;      // 16 waves: four per SIMD hide the LDS and issue latencies of the short loop body
constexpr int SS_WAVES = SS_THREADS / 64;
constexpr int SS_LOADERS = 4;        // waves 0 .. 3 issue the asynchronous copies (8 x 4 rows each per block)
constexpr int SS_PROTO = 4;          // this wave collects the siblings' min / max (loads only, so that its waits
                                     // for a poll never include a store on its way to memory)
constexpr int SS_WRITER = 5;         // this wave publishes the workgroup's min / max and writes sigma out
constexpr int SS_BR = 128;           // rows per block: two rows per thread and iteration, so that the scalar
                                     // bookkeeping of an iteration is paid once per 32 KB
constexpr int SS_BLOCK_BYTES = SS_BR * 256;
constexpr int SS_NSLOT = 4;          // LDS ring, blocks (128 KB)
// Blocks in flight ahead of the one whose min / max are taken (PF) and blocks between taking a block's min / max
// and scoring it (LAG): PF + LAG + 1 ring slots.  Workgroups that exchange need the LAG to cover the exchange;
// a workgroup that owns whole chunks (W = 1) has its min / max at once and spends the ring on copies in flight.
constexpr int SS_LAG_X = 2, SS_PF_X = 1;     // W > 1
constexpr int SS_LAG_1 = 1, SS_PF_1 = 2;     // W = 1
constexpr int SS_LAG_MAX = SS_LAG_X;         // the larger of the two: sizes the mailbox ring and the slices
constexpr int SS_NR = 8;             // mailbox ring over chunks
static_assert(SS_NR >= SS_LAG_MAX + 2 && (SS_NR & (SS_NR - 1)) == 0, "a sibling runs at most SS_LAG_MAX + 1 chunks ahead");
constexpr int SS_MAX_WGS = 256;      // workgroups that exchange (W > 1): one per CU
constexpr int SS_MAX_W = 2;          // siblings per (stream, range)
constexpr int SS_MAX_CHUNKS = 4095;  // the chunk index is 12 bits of the tag
constexpr int SS_SPIN = 2048;        // polls before a reader stops waiting for a mailbox

typedef unsigned long long mail_t;
constexpr size_t SS_MAIL_WORDS = size_t(SS_MAX_WGS) * SS_NR * 128;
// words [workgroup][chunk & 7][channel]
static __device__ __align__(256) mail_t g_mail_part[SS_MAIL_WORDS];

struct StreamPlan {
    int use;        // the streaming kernel applies
    int nstreams;   // B * Hkv * 2
    int ranges;     // chunk ranges per stream
    int cpr;        // scored chunks per range (the last range may hold fewer)
    int W;          // row slices (sibling workgroups) per (stream, range): a power of two
    int R;          // rows of a chunk per sibling
    int nblk;       // blocks of SS_BR rows per sibling and chunk
    int wgs;        // nstreams * ranges * W
};

static StreamPlan make_stream_plan(const Dims& D, int cus) {
    StreamPlan P = {};
    P.nstreams = D.B * D.Hkv * 2;
    P.use = D.dtype == 1 && D.d == 128 && D.Ns > 0 && D.Ns + 1 <= SS_MAX_CHUNKS && D.L <= FUSED_MAX_L &&
            D.ks[2] % 8 == 0 && D.ks[2] <= (int64_t(1) << 22);
    if (!P.use) return P;
    const int slots = cus < SS_MAX_WGS ? cus : SS_MAX_WGS;
    int W = 1, ranges = 1;
    auto fits = [&](int w_, int r_) { return int64_t(P.nstreams) * w_ * r_ <= slots; };
    auto slice_ok = [&](int w_) { return D.L / w_ >= SS_LAG_MAX * SS_BR; };   // a slice holds >= SS_LAG_MAX blocks
    while (fits(W, ranges + 1) && D.Ns / (ranges + 1) >= 8) ++ranges;
    while (W < SS_MAX_W && fits(W * 2, ranges) && slice_ok(W * 2)) W *= 2;
    while (fits(W, ranges + 1) && D.Ns / (ranges + 1) >= 6) ++ranges;
    int R = (D.L + W - 1) / W;
    while (W > 1 && (W - 1) * R >= D.L) { W /= 2; R = (D.L + W - 1) / W; }   // every sibling owns a row
    P.cpr = (D.Ns + ranges - 1) / ranges;
    P.ranges = (D.Ns + P.cpr - 1) / P.cpr;
    P.W = W;
    P.R = R;
    P.nblk = (R + SS_BR - 1) / SS_BR;
    P.wgs = P.nstreams * P.ranges * W;
    // Worth it only when the cut fills most of the chip and reads little twice (each range re-reads one chunk);
    // otherwise (few KV heads, short sequences) the one-workgroup-per-chunk kernel is the faster one.
    const bool fills = int64_t(P.wgs) * 4 >= int64_t(slots) * 3;
    const bool lean = int64_t(D.Ns + P.ranges) * 100 <= int64_t(D.Ns + 1) * 115;
    P.use = fills && lean;
    return P;
}

// ---- packed 16-bit min / max: bf16 patterns of finite values below 2^121 order like 16-bit floats ---------------
__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b) {
    uint32_t d;
    asm("v_pk_min_f16 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
    return d;
}
__device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b) {
    uint32_t d;
    asm("v_pk_max_f16 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
    return d;
}
constexpr uint32_t PK_POS_INF = 0x7c007c00u, PK_NEG_INF = 0xfc00fc00u;   // identities of pk_min / pk_max

struct MinMax8 {   // running min / max of 8 channels (one 16-byte piece of a row)
    uint32_t mn[4], mx[4];
    __device__ __forceinline__ void reset() {
#pragma unroll
        for (int i = 0; i < 4; ++i) { mn[i] = PK_POS_INF; mx[i] = PK_NEG_INF; }
    }
    __device__ __forceinline__ void take(const uint4& v) {
        mn[0] = pk_min(mn[0], v.x); mn[1] = pk_min(mn[1], v.y); mn[2] = pk_min(mn[2], v.z); mn[3] = pk_min(mn[3], v.w);
        mx[0] = pk_max(mx[0], v.x); mx[1] = pk_max(mx[1], v.y); mx[2] = pk_max(mx[2], v.z); mx[3] = pk_max(mx[3], v.w);
    }
    __device__ __forceinline__ void merge(const uint32_t (&omn)[4], const uint32_t (&omx)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { mn[i] = pk_min(mn[i], omn[i]); mx[i] = pk_max(mx[i], omx[i]); }
    }
};

__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// one mailbox word {tag : 32, max : bf16, min : bf16} is written as a single 8-byte store
__device__ __forceinline__ void mail_store(mail_t* p, mail_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 64 lanes x 16 bytes of mailbox words -> LDS, as a device-scope load (the level at which a sibling's store is seen)
__device__ __forceinline__ void mail_fetch16(const mail_t* src, unsigned lds_byte_addr) {
    const unsigned la = __builtin_amdgcn_readfirstlane(lds_byte_addr);
    unsigned keep;
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off sc1\n\ts_mov_b32 m0, %0"
        : "=&s"(keep)
        : "v"(src), "s"(la)
        : "memory");
}

// one asynchronous copy of 64 x 16 bytes to the LDS byte address `lds_byte_addr` (wave-uniform)
__device__ __forceinline__ void async_copy16_to(const void* src, unsigned lds_byte_addr) {
    const unsigned la = __builtin_amdgcn_readfirstlane(lds_byte_addr);
    unsigned keep;
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
        : "=&s"(keep)
        : "v"(src), "s"(la)
        : "memory");
}

// The four copies of one block that a loader wave makes (64 x 16 bytes each, 1 KB apart in LDS): the LDS address
// register M0 is set once and stepped, the global base is wave-uniform, the lanes bring 32-bit byte offsets.
__device__ __forceinline__ void async_block4(const void* base, unsigned v0, unsigned v1, unsigned v2, unsigned v3,
                                             unsigned lds_byte_addr) {
    const unsigned la = __builtin_amdgcn_readfirstlane(lds_byte_addr);
    const unsigned long long b = (unsigned long long)(size_t)base;
    const unsigned blo = __builtin_amdgcn_readfirstlane((unsigned)b), bhi = __builtin_amdgcn_readfirstlane((unsigned)(b >> 32));
    const unsigned long long sb = (unsigned long long)blo | ((unsigned long long)bhi << 32);
    unsigned keep;   // M0 is saved and restored around the block
    asm volatile(
        "s_mov_b32 %0, m0\n\t"
        "s_mov_b32 m0, %6\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %5\n\t"
        "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %5\n\t"
        "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %3, %5\n\t"
        "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %4, %5\n\t"
        "s_mov_b32 m0, %0"
        : "=&s"(keep)
        : "v"(v0), "v"(v1), "v"(v2), "v"(v3), "s"(sb), "s"(la)
        : "memory", "scc");
}

struct StreamLds {
    unsigned char ring[SS_NSLOT * SS_BLOCK_BYTES];
    uint32_t red[2][SS_WAVES][16][8];   // per wave and 16-byte column: 4 words of packed min, 4 of packed max
    uint32_t own[SS_NR][128];           // this workgroup's min / max of a chunk, per channel: max16 << 16 | min16
    float coef_a[2][128], coef_b[2][128];
    float stage[2][SS_BR];              // standard deviations of one block on their way to global memory
    mail_t poll[SS_MAX_W - 1][128];     // landing zone of the siblings' words
    uint32_t comb[2][128];              // min / max of a whole chunk (max16 << 16 | min16), by chunk parity
    int ready[2];
};

// Workgroup barrier that also completes this wave's LDS writes first (the bare ring_barrier() does not: it is
// meant for data that arrives by asynchronous copies).  No vector-memory wait, so copies stay in flight.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Eq. 6 as one fused multiply-add per value: a = 1 / den, b = -min / den - 1/2
__device__ __forceinline__ void coef_from_word(uint32_t w, float& a, float& b) {
    const float mn = bf16lo(w), mx = bf16hi(w);
    float den = mx - mn;
    den = den == 0.0f ? 1.0f : den;
    a = 1.0f / den;
    b = __builtin_fmaf(-mn, a, -0.5f);
}

template <int SS_PF, int SS_LAG>   // copies in flight, blocks between min / max and scoring
__global__ __launch_bounds__(SS_THREADS, 1) void k_score_stream(Dims D, const bf16_t* __restrict__ Kp,
                                                                 const bf16_t* __restrict__ Vp,
                                                                 float* __restrict__ sigma, mail_t* mail_part,
                                                                 StreamPlan P, uint32_t tagbase) {
    static_assert(SS_PF + SS_LAG + 1 <= SS_NSLOT, "a ring slot is refilled only after its block has been scored");
    __shared__ __attribute__((aligned(1024))) StreamLds sh;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int W = P.W, nblk = P.nblk;
    const int wg = blockIdx.x;
    const int w = wg % W, sr = wg / W;            // sibling, (stream, range)
    const int range = sr % P.ranges, s = sr / P.ranges;
    const int z = s & 1, bh = s >> 1, b = bh / D.Hkv, h = bh % D.Hkv;
    const bf16_t* Z = (z ? Vp : Kp) + b * D.ks[0] + h * D.ks[1];
    // scored chunks [p0, p1) of this range; the walk starts at chunk p1 (reference only) and ends at p0
    const int p0 = range * P.cpr, p1 = min(D.Ns, p0 + P.cpr);
    const int T = (p1 - p0 + 1) * nblk;          // blocks of this workgroup
    const int r_begin = w * P.R, r_end = min(r_begin + P.R, D.L);
    const float inv_d = 1.0f / 128.0f, inv_dof = 1.0f / float(128 - D.ddof);
    // LDS byte addresses: the low half of a generic pointer into LDS is the offset inside LDS
    const unsigned ring_la = unsigned(reinterpret_cast<size_t>(&sh.ring[0])), poll_la = unsigned(reinterpret_cast<size_t>(&sh.poll[0][0]));

    // The blocks of the walk are numbered 0 .. T-1: block t is rows j * SS_BR .. of this slice of chunk p1 - t / nblk,
    // j = t % nblk.  Every cursor below keeps its (chunk, j, ring slot) by counting, never by dividing.
    struct Cursor {
        int c, j, slot;
    };
    Cursor ld = {p1, 0, 0};                       // next block to copy in
    // First row (within the slice) of block j.  A slice of at least one block: the last block is moved back so
    // that it ends with the slice (rows it shares with the block before are scored twice, to the same values);
    // a shorter slice: one block, rows past the slice repeat its last row.
    const int rows = r_end - r_begin;
    const bool whole_blocks = rows >= SS_BR;
    auto block_row0 = [&](int j) { return whole_blocks ? min(j * SS_BR, rows - SS_BR) : 0; };
    // per-lane byte offsets of the loader's eight copies inside a block (rows 32*wave + 4k + lane/16)
    unsigned lane_off[8];
#pragma unroll
    for (int k = 0; k < 8; ++k)
        lane_off[k] = unsigned(((32 * wave + 4 * k + (lane >> 4)) * D.ks[2] + (lane & 15) * 8) * 2);
    const int64_t chunk_bytes = int64_t(D.L) * D.ks[2] * 2;
    const unsigned row_bytes = unsigned(D.ks[2] * 2);
    // slice start of the chunk the loader is in
    const unsigned char* ld_base = reinterpret_cast<const unsigned char*>(Z + (int64_t(D.S) + int64_t(p1) * D.L + r_begin) * D.ks[2]);
    auto issue = [&]() {
        // past the end (ld.c < p0): repeat the last block into the slot in turn (never used), so that every
        // iteration issues the same number of copies and one vmcnt value names a block
        const int j = ld.c < p0 ? nblk - 1 : ld.j;
        const unsigned char* src = ld_base + (ld.c < p0 ? chunk_bytes : 0) + unsigned(block_row0(j)) * row_bytes;
        const unsigned dst = ring_la + ld.slot * SS_BLOCK_BYTES + wave * 8192;
        if (whole_blocks) {
            async_block4(src, lane_off[0], lane_off[1], lane_off[2], lane_off[3], dst);
            async_block4(src, lane_off[4], lane_off[5], lane_off[6], lane_off[7], dst + 4096);
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int rloc = min(32 * wave + 4 * k + (lane >> 4), rows - 1);
                async_copy16_to(src + (int64_t(rloc) * D.ks[2] + (lane & 15) * 8) * 2, dst + k * 1024);
            }
        }
        if (ld.c >= p0) {
            ld.j += 1;
            if (ld.j == nblk) { ld.j = 0; ld.c -= 1; ld_base -= chunk_bytes; }
        }
        ld.slot = ld.slot + 1 == SS_NSLOT ? 0 : ld.slot + 1;
    };

    // this thread's 16-byte piece (8 channels) of rows r and r + 64 of a block: the 16 lanes of a row read 256
    // contiguous bytes
    const int r = tid >> 4, o = tid & 15;
    const int offA = r * 256 + o * 16, offB = offA + 64 * 256;

    MinMax8 mA;
    mA.reset();
    float a[8], bq[8];     // Eq. 6 coefficients of this thread's channels
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = 0.0f; bq[e] = 0.0f; }

    // protocol state (wave SS_PROTO)
    int pub_c = p1 + 1;          // chunks >= pub_c have been published
    int ex_c = p1;               // chunk whose siblings' words are being collected (down to p0 + 1)
    int ex_done_c = p1 + 1;      // chunks >= ex_done_c are complete (their words are in sh.comb)
    unsigned ex_have = 0;        // siblings of ex_c already merged
    int ex_issued = 0;
    float ex_mn0 = 0.0f, ex_mx0 = 0.0f, ex_mn1 = 0.0f, ex_mx1 = 0.0f;   // channels 2*lane, 2*lane + 1 so far
    const uint32_t seq_tag = tagbase;
    mail_t* my_part = mail_part + size_t(wg) * SS_NR * 128;
    const mail_t* sib_part = mail_part + size_t(sr) * W * SS_NR * 128;
    const unsigned ex_all = ((1u << W) - 1u) & ~(1u << w);

    // ---- protocol pieces, run by wave SS_PROTO only --------------------------------------------------------
    // this workgroup's min / max of chunk c from the per-wave records of buffer `buf`: words of channels 2*lane, +1
    auto own_words = [&](int buf, uint32_t& w0, uint32_t& w1) {
        const int col = lane >> 2, wd = lane & 3;
        uint32_t mn = PK_POS_INF, mx = PK_NEG_INF;
#pragma unroll
        for (int wv = 0; wv < SS_WAVES; ++wv) {
            mn = pk_min(mn, sh.red[buf][wv][col][wd]);
            mx = pk_max(mx, sh.red[buf][wv][col][4 + wd]);
        }
        w0 = ((mx & 0xffffu) << 16) | (mn & 0xffffu);
        w1 = (mx & 0xffff0000u) | (mn >> 16);
    };
    auto finish_own = [&](int c, int buf) {                // wave SS_PROTO: keep them for the exchange
        uint32_t w0, w1;
        own_words(buf, w0, w1);
        sh.own[c & (SS_NR - 1)][2 * lane] = w0;
        sh.own[c & (SS_NR - 1)][2 * lane + 1] = w1;
        pub_c = c;
    };
    auto publish_own = [&](int c, int buf) {               // wave SS_WRITER: into the mailbox
        if (W == 1 || c <= p0) return;                     // the min / max of chunk p0 serve nobody
        uint32_t w0, w1;
        own_words(buf, w0, w1);
        const uint32_t tag = seq_tag | uint32_t(c);
        mail_t* dst = my_part + (c & (SS_NR - 1)) * 128 + 2 * lane;
        mail_store(dst, (mail_t(tag) << 32) | w0);
        mail_store(dst + 1, (mail_t(tag) << 32) | w1);
    };
    // one step of the exchange: merge what the last polls brought, poll again for what is missing
    auto exch_step = [&]() {
        if (W == 1 || ex_c <= p0 || ex_c < pub_c) return;   // nothing to collect, or own words not out yet
        const int slot = ex_c & (SS_NR - 1);
        if (ex_issued) {
            wait_vmcnt<0>();
            const uint32_t tag = seq_tag | uint32_t(ex_c);
            for (int k = 0; k < W; ++k) {
                if (!((ex_all & ~ex_have) >> k & 1u)) continue;
                const mail_t* pz = sh.poll[k < w ? k : k - 1];
                const mail_t q0 = pz[2 * lane], q1 = pz[2 * lane + 1];
                const bool ok = uint32_t(q0 >> 32) == tag && uint32_t(q1 >> 32) == tag;
                if (__builtin_amdgcn_ballot_w64(!ok) != 0) continue;
                ex_mn0 = fminf(ex_mn0, bf16lo(uint32_t(q0))); ex_mx0 = fmaxf(ex_mx0, bf16hi(uint32_t(q0)));
                ex_mn1 = fminf(ex_mn1, bf16lo(uint32_t(q1))); ex_mx1 = fmaxf(ex_mx1, bf16hi(uint32_t(q1)));
                ex_have |= 1u << k;
            }
            ex_issued = 0;
        } else {
            const uint32_t o0 = sh.own[slot][2 * lane], o1 = sh.own[slot][2 * lane + 1];
            ex_mn0 = bf16lo(o0); ex_mx0 = bf16hi(o0);
            ex_mn1 = bf16lo(o1); ex_mx1 = bf16hi(o1);
        }
        if (ex_have == ex_all) {
            sh.comb[ex_c & 1][2 * lane] = (__float_as_uint(ex_mx0) & 0xffff0000u) | (__float_as_uint(ex_mn0) >> 16);
            sh.comb[ex_c & 1][2 * lane + 1] = (__float_as_uint(ex_mx1) & 0xffff0000u) | (__float_as_uint(ex_mn1) >> 16);
            ex_done_c = ex_c;
            ex_c -= 1;
            ex_have = 0;
            return;                                          // the next chunk's own words come at least a block later
        }
        for (int k = 0; k < W; ++k)
            if ((ex_all & ~ex_have) >> k & 1u)
                mail_fetch16(sib_part + (size_t(k) * SS_NR + slot) * 128 + 2 * lane, poll_la + (k < w ? k : k - 1) * 1024);
        ex_issued = 1;
    };
    // Eq. 6 coefficients for scoring chunk c into buffer `buf`: true when they are in place
    auto coef_try = [&](int c, int buf) -> bool {
        const int c1 = c + 1;
        uint32_t w0, w1;
        if (W == 1) {
            w0 = sh.own[c1 & (SS_NR - 1)][2 * lane];
            w1 = sh.own[c1 & (SS_NR - 1)][2 * lane + 1];
        } else {
            if (ex_done_c > c1) return false;
            w0 = sh.comb[c1 & 1][2 * lane];
            w1 = sh.comb[c1 & 1][2 * lane + 1];
        }
        float a0, b0, a1, b1;
        coef_from_word(w0, a0, b0);
        coef_from_word(w1, a1, b1);
        sh.coef_a[buf][2 * lane] = a0; sh.coef_b[buf][2 * lane] = b0;
        sh.coef_a[buf][2 * lane + 1] = a1; sh.coef_b[buf][2 * lane + 1] = b1;
        return true;
    };
    // standard deviations of the block (c, j), staged in buffer `buf` -> global memory
    auto write_out = [&](int c, int j, int buf) {
        float* dst = sigma + (int64_t(s) * D.Ns + c) * D.L;
        const int rloc = r_begin + block_row0(j) + lane;
        if (rloc < r_end) dst[rloc] = sh.stage[buf][lane];
        if (rloc + 64 < r_end) dst[rloc + 64] = sh.stage[buf][lane + 64];
    };

    // ---- the walk ----------------------------------------------------------------------------------------------
    // Iteration i takes the min / max of block i (chunk index ci = i / nblk, block j = i % nblk) and scores block
    // i - SS_LAG.  Two nested loops so that the per-block control is a handful of scalar operations: the scored
    // block starts a chunk exactly when j == js, and its coefficients are prepared one iteration earlier (j == jp).
    if (wave < SS_LOADERS)
        for (int blk = 0; blk < SS_PF; ++blk) issue();
    const int iters = T + SS_LAG;
    const int nch = p1 - p0 + 1;                                 // chunks of the walk, the reference-only top one included
    const int js = SS_LAG % nblk, jp = (js + nblk - 1) % nblk, dq = SS_LAG / nblk;
    int sci = -dq - 1;                                           // chunk index (0 = top) of the block being scored
    int sj = 0;                                                  // ... and its block index in the chunk
    bool sg_on = false;                                          // the scored block belongs to a scored chunk
    int mm_off = 0, sg_off = ((SS_NSLOT - SS_LAG % SS_NSLOT) % SS_NSLOT) * SS_BLOCK_BYTES;   // ring offsets of the two blocks
    int prev_on = 0, prev_c = 0, prev_j = 0;                     // what the previous iteration scored
    int mm_ended = 0;                                            // the previous iteration closed a chunk's min / max
    int i = 0;
    for (int ci = 0; i < iters; ++ci) {
      const bool mm_on = ci < nch;
      for (int j = 0; j < nblk && i < iters; ++j, ++i) {
        if (wave < SS_LOADERS) wait_vmcnt<8 * (SS_PF - 1)>();   // this wave's copies of block i have landed
        lds_barrier();
        if (wave < SS_LOADERS) issue();
        bool sg_start = false;
        if (j == js) {                                           // the scored block enters the next chunk
            sci += 1;
            sj = 0;
            sg_on = sci >= 1 && sci < nch;                       // index 0 is the reference-only top chunk
            sg_start = sg_on;
        }
        if (wave == SS_WRITER) {
            if (mm_ended) publish_own(p1 - (ci - 1), (i - 1) & 1);
            if (prev_on) write_out(prev_c, prev_j, (i - 1) & 1);
        }
        if (wave == SS_PROTO) {
            if (mm_ended) finish_own(p1 - (ci - 1), (i - 1) & 1);
            exch_step();
            if (j == jp && sci + 1 >= 1 && sci + 1 < nch && i + 1 < iters) {   // next iteration starts a scored chunk
                const int nc = p1 - (sci + 1), buf = nc & 1;
                const bool ok = coef_try(nc, buf);
                if (lane == 0) sh.ready[buf] = ok ? 1 : 0;
            }
        }
        mm_ended = 0;
        if (sg_start) {
            const int c = p1 - sci, buf = c & 1;
            int ok = sh.ready[buf];
            // Not in place (a sibling is late): wait, helping the siblings meanwhile.  Two barriers per try so that
            // every wave reads the same flag.
            for (int tries = 0; !ok && tries < SS_SPIN; ++tries) {
                lds_barrier();
                if (wave == SS_PROTO) {
                    __builtin_amdgcn_s_sleep(2);
                    exch_step();
                    const bool got = coef_try(c, buf);
                    if (lane == 0) sh.ready[buf] = got ? 1 : 0;
                }
                lds_barrier();
                ok = sh.ready[buf];
            }
            if (!ok) {
                // The mailboxes did not deliver: min / max of chunk c + 1 from its rows (every thread: one 16-byte
                // column, rows tid / 16, + 32, ...).
                lds_barrier();
                MinMax8 f;
                f.reset();
                const int64_t row0 = int64_t(D.S) + int64_t(c + 1) * D.L;
                for (int rr = tid >> 4; rr < D.L; rr += SS_THREADS / 16)
                    f.take(*reinterpret_cast<const uint4*>(Z + (row0 + rr) * D.ks[2] + (tid & 15) * 8));
#pragma unroll
                for (int off = 16; off < 64; off <<= 1) {
                    uint32_t omn[4], omx[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) { omn[k] = __shfl_xor(f.mn[k], off, 64); omx[k] = __shfl_xor(f.mx[k], off, 64); }
                    f.merge(omn, omx);
                }
                // the per-wave records of buffer i & 1 are free here: this iteration's own records come later
                if (lane < 16) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) { sh.red[i & 1][wave][lane][k] = f.mn[k]; sh.red[i & 1][wave][lane][4 + k] = f.mx[k]; }
                }
                __syncthreads();
                if (wave == SS_PROTO) {
                    const int col = lane >> 2, wd = lane & 3;
                    uint32_t mn = PK_POS_INF, mx = PK_NEG_INF;
#pragma unroll
                    for (int wv = 0; wv < SS_WAVES; ++wv) {
                        mn = pk_min(mn, sh.red[i & 1][wv][col][wd]);
                        mx = pk_max(mx, sh.red[i & 1][wv][col][4 + wd]);
                    }
                    float a0, b0, a1, b1;
                    coef_from_word(((mx & 0xffffu) << 16) | (mn & 0xffffu), a0, b0);
                    coef_from_word((mx & 0xffff0000u) | (mn >> 16), a1, b1);
                    sh.coef_a[buf][2 * lane] = a0; sh.coef_b[buf][2 * lane] = b0;
                    sh.coef_a[buf][2 * lane + 1] = a1; sh.coef_b[buf][2 * lane + 1] = b1;
                    if (ex_c == c + 1) {      // give the exchange of this chunk up: its result is no longer needed
                        wait_vmcnt<0>();
                        ex_done_c = ex_c; ex_c -= 1; ex_have = 0; ex_issued = 0;
                    }
                }
                __syncthreads();
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) { a[e] = sh.coef_a[buf][8 * o + e]; bq[e] = sh.coef_b[buf][8 * o + e]; }
        }
        // ---- min / max of block i
        if (mm_on) {
            const unsigned char* src = sh.ring + mm_off;
            mA.take(*reinterpret_cast<const uint4*>(src + offA));
            mA.take(*reinterpret_cast<const uint4*>(src + offB));
            if (j + 1 == nblk) {
                mm_ended = 1;
                // end of a chunk: the four rows of a wave (lanes 16, 32 apart), then one record per wave
#pragma unroll
                for (int off = 16; off < 64; off <<= 1) {
                    uint32_t omn[4], omx[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) { omn[k] = __shfl_xor(mA.mn[k], off, 64); omx[k] = __shfl_xor(mA.mx[k], off, 64); }
                    mA.merge(omn, omx);
                }
                if (lane < 16) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) { sh.red[i & 1][wave][o][k] = mA.mn[k]; sh.red[i & 1][wave][o][4 + k] = mA.mx[k]; }
                }
                mA.reset();
            }
        }
        // ---- standard deviation over the channels of the rows of block sg (Eq. 6-7)
        if (sg_on) {
            const unsigned char* src = sh.ring + sg_off;
            // Std over the 128 channels of one row from this lane's 8 values (Eq. 6-7); the 16 lanes of the row
            // get the same result
            auto row_sigma = [&](const uint4& v) {
                const uint32_t wsrc[4] = {v.x, v.y, v.z, v.w};
                float x[8];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    x[2 * k] = __builtin_fmaf(bf16lo(wsrc[k]), a[2 * k], bq[2 * k]);
                    x[2 * k + 1] = __builtin_fmaf(bf16hi(wsrc[k]), a[2 * k + 1], bq[2 * k + 1]);
                }
                float s1 = x[0] + x[1], s2 = x[0] * x[0];
                s2 = __builtin_fmaf(x[1], x[1], s2);
#pragma unroll
                for (int e = 2; e < 8; ++e) {
                    s1 += x[e];
                    s2 = __builtin_fmaf(x[e], x[e], s2);
                }
                s1 = row16_sum(s1);
                s2 = row16_sum(s2);
                const float m2 = s1 * s1 * inv_d;
                float var = s2 - m2;
                if (__builtin_amdgcn_ballot_w64(m2 > 0.25f * s2) != 0) {     // the two terms cancel: from the deviations
                    const float mean = s1 * inv_d;
                    float q = 0.0f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) { const float dv = x[e] - mean; q = __builtin_fmaf(dv, dv, q); }
                    var = row16_sum(q);
                }
                return __builtin_amdgcn_sqrtf(fmaxf(var, 0.0f) * inv_dof);
            };
            const uint4 vA = *reinterpret_cast<const uint4*>(src + offA);
            const uint4 vB = *reinterpret_cast<const uint4*>(src + offB);
            const float sgA = row_sigma(vA), sgB = row_sigma(vB);
            if (o == 0) { sh.stage[i & 1][r] = sgA; sh.stage[i & 1][r + 64] = sgB; }
        }
        if (wave == SS_PROTO && ex_issued) exch_step();   // a second look at the polls within the iteration
        prev_on = sg_on ? 1 : 0;
        prev_c = p1 - sci;
        prev_j = sj;
        sj += 1;
        mm_off = mm_off + SS_BLOCK_BYTES == SS_NSLOT * SS_BLOCK_BYTES ? 0 : mm_off + SS_BLOCK_BYTES;
        sg_off = sg_off + SS_BLOCK_BYTES == SS_NSLOT * SS_BLOCK_BYTES ? 0 : sg_off + SS_BLOCK_BYTES;
      }
    }
    // the last block's standard deviations
    if (wave < SS_LOADERS) wait_vmcnt<0>();   // copies issued past the end land before the LDS is released
    __syncthreads();
    if (wave == SS_WRITER && prev_on) write_out(prev_c, prev_j, (iters - 1) & 1);
    if (wave == SS_PROTO && W > 1) wait_vmcnt<0>();   // polls still in flight
}

// Softmax over the chunk's tokens for K and V, summed (Eq. 7-8); SELECT: the chunk's top K right away (text after
// Eq. 8).  One workgroup of NT threads per (batch, KV head, chunk).  The work is a chain of short block-wide
// reductions and scans: with many chunks small workgroups (several per CU) finish soonest, with few chunks (fewer
// than CUs) the chain itself is the time and more threads shorten it.  Dynamic LDS: 2 * L floats.  The workgroups
// also clear the mailbox words that the streaming kernel of this call may have written.
template <bool SELECT, int NT>
__global__ __launch_bounds__(NT) void k_softmax_select(Dims D, const float* __restrict__ sigma, float* __restrict__ score,
                                                       int32_t* __restrict__ idx, mail_t* mail_part, int part_words) {
    const int p = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
    extern __shared__ float sx_sig[];     // [2][L]
    __shared__ float sm[NT / 64];
    float* sig0 = sx_sig;
    float* sig1 = sx_sig + D.L;
    const float* sk = sigma + ((int64_t(bh) * 2 + 0) * D.Ns + p) * D.L;
    const float* sv = sigma + ((int64_t(bh) * 2 + 1) * D.Ns + p) * D.L;
    for (int r = tid; r < D.L; r += NT) { sig0[r] = sk[r]; sig1[r] = sv[r]; }
    __syncthreads();
    softmax_sum_block<NT>(sig0, sig1, sm, D.L, score + (int64_t(bh) * D.Ns + p) * D.L);
    if (SELECT) {
        __shared__ SelectLds sel;
        __syncthreads();
        select_topk_block<NT>(reinterpret_cast<const uint32_t*>(sig0), D.L, D.K, D.S + p * D.L,
                              idx + (int64_t(bh) * D.Ns + p) * D.K, sel);
    }
    const int64_t g = int64_t(bh) * gridDim.x + p, G = int64_t(gridDim.x) * gridDim.y;
    for (int64_t e = g * NT + tid; e < part_words; e += G * NT) mail_part[e] = 0;
}

static hipError_t run_softmax_select(const Dims& D, const float* sigma, float* score, int32_t* idx, mail_t* mail,
                                     int part_words, hipStream_t st) {
    const size_t lds = size_t(2) * D.L * sizeof(float);
    const dim3 grid(D.Ns, D.B * D.Hkv);
    const bool few = int64_t(D.Ns) * D.B * D.Hkv <= 128 && D.L >= 1024;
#define LRSA_SX(name, SEL, NT_) \
    LRSA_TIMED_LAUNCH(name, st, (k_softmax_select<SEL, NT_>), grid, dim3(NT_), lds, st, D, sigma, score, idx, mail, part_words)
    if (idx) { if (few) LRSA_SX("k_softmax_select", true, 1024); else LRSA_SX("k_softmax_select", true, 256); }
    else { if (few) LRSA_SX("k_softmax", false, 1024); else LRSA_SX("k_softmax", false, 256); }
#undef LRSA_SX
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ host side
namespace {
struct DeviceState {
    mail_t* part = nullptr;
    int cus = 0;
};
std::mutex g_mu;
DeviceState g_dev[64];
std::atomic<uint32_t> g_seq{0};

// mailbox addresses on the current device and its CU count, looked up once per device
hipError_t device_state(DeviceState* out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_mu);
    DeviceState& st = g_dev[dev];
    if (!st.part) {
        void* pp = nullptr;
        int cus = 0;
        if ((e = hipGetSymbolAddress(&pp, HIP_SYMBOL(g_mail_part))) != hipSuccess) return e;
        if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
        if (!pp) return hipErrorInvalidSymbol;
        st.cus = cus;
        st.part = static_cast<mail_t*>(pp);
    }
    *out = st;
    return hipSuccess;
}
}  // namespace

// Eq. 7-8 (and the selection when idx is given) from standard deviations that other kernels left in `sigma`
hipError_t launch_softmax_select(const Dims& D, const float* sigma, float* score, int32_t* idx, hipStream_t st) {
    return run_softmax_select(D, sigma, score, idx, nullptr, 0, st);
}

bool score_stream_applies(const Dims& D) { return make_stream_plan(D, SS_MAX_WGS).use != 0; }

// scores (and, with idx, the selection) through the streaming kernel; sigma: B * Hkv * 2 * Ns * L floats of workspace
hipError_t launch_score_stream(const Dims& D, const void* K, const void* V, float* score, int32_t* idx, float* sigma,
                               hipStream_t st) {
    DeviceState ds;
    const hipError_t e = device_state(&ds);
    if (e != hipSuccess) return e;
    const StreamPlan P = make_stream_plan(D, ds.cus);
    const uint32_t seq = g_seq.fetch_add(1) % 0xfffffu + 1u;          // 1 .. 2^20 - 1: a tag is never zero
    if (P.W > 1)
        LRSA_TIMED_LAUNCH("k_score_stream", st, (k_score_stream<SS_PF_X, SS_LAG_X>), dim3(P.wgs), dim3(SS_THREADS), 0, st, D,
                          (const bf16_t*)K, (const bf16_t*)V, sigma, ds.part, P, seq << 12);
    else
        LRSA_TIMED_LAUNCH("k_score_stream", st, (k_score_stream<SS_PF_1, SS_LAG_1>), dim3(P.wgs), dim3(SS_THREADS), 0, st, D,
                          (const bf16_t*)K, (const bf16_t*)V, sigma, ds.part, P, seq << 12);
    const int part_words = P.W > 1 ? P.wgs * SS_NR * 128 : 0;
    return run_softmax_select(D, sigma, score, idx, ds.part, part_words, st);
}

}  // namespace lrsa
