// One-read LagKV scoring for bf16 data with head_dim 128 (Eq. 4-8 of the paper): every K and V row is read
// from memory ONCE, by the workgroup that keeps it in registers until it has been scored.
//
// Eq. 6 normalises chunk p with the per-channel min / max of chunk p+1 (Eq. 4-5): a row takes part in the min / max
// of its own chunk and, normalised with the statistics of the NEXT chunk, in its own standard deviation (Eq. 7).
// A *stream* is one (batch, KV head, K or V) tensor.  A workgroup of NT threads loads NT rows of ONE chunk of one
// stream into registers (16 pieces of 16 bytes per thread) and keeps them there.  It takes their per-channel
// min / max, publishes them as *mailbox words* for the workgroups of the chunk below, collects the words of all
// parts of the chunk above (its reference) and then scores its rows out of the registers.  A chunk of L rows is cut
// into W = ceil(L / NT) parts (the last one is moved back so that it ends with the chunk: the rows it shares with
// the part before get the same values from both).  The grid is ordered by descending chunk, so the workgroups a
// reader waits for were dispatched before it and wait for nobody that comes after them.
//
// Mailboxes live in device memory that belongs to the library:
//   * a word is {tag : 32, max : bf16, min : bf16} of one channel, written and read as ONE 8-byte access; the tag
//     names the call and the chunk, so a reader knows whether the word it sees is the one it wants;
//   * a workgroup publishes the 128 words of its part into the slot `its index in the grid modulo SR_MAIL_SLOTS`.
//     A reader and its writers are nstreams * W (+- W) workgroups apart; two workgroups that share a slot are
//     SR_MAIL_SLOTS apart and, the plan sees to it, belong to different chunks, so their tags differ;
//   * the mailboxes are hints only: a reader that does not find its tags within its poll limit computes the min / max
//     of the reference chunk from the rows themselves.  Whatever the mailboxes hold, results are the same.
// Several small workgroups share a CU: the loads of a CU return in the order they were issued, so the first
// workgroup scores while the data of the next ones is still arriving.
//
// A second kernel takes the softmax over each chunk's tokens for K and V, adds them (Eq. 7-8), optionally
// selects the top K (text after Eq. 8), and clears the mailboxes the call used.
//
// Arithmetic: min / max are exact (packed 16-bit compares on the stored bf16 patterns); Eq. 6 is evaluated as
// z * (1 / den) - min / den, shifted by 1/2 so that the normalised values centre on zero; the variance over
// the channels is sum(x^2) - sum(x)^2 / d in fp32 and is recomputed from the deviations for a row in which the two
// terms cancel.  Values of magnitude >= 2^121 or NaN are outside the contract (their bf16 patterns do not order
// like numbers in a 16-bit float compare).
#include "score_block.h"
#include "select_block.h"

#include <atomic>
#include <mutex>

namespace lrsa {

constexpr int SR_MAX_PARTS = 16;     // parts per chunk: the bits of a reader's "have" mask
constexpr int SR_SPIN = 256;         // polls before a reader stops waiting for a mailbox (the default of lrsa_score_poll_limit):
                                     // a writer's words are usually there at the first or second look; 256 looks are about a
                                     // millisecond, after which a second read of the chunk is the cheaper way
constexpr int SR_MAX_CHUNKS = 4095;  // the chunk index is 12 bits of the tag
constexpr int SR_MAIL_SLOTS = 8192;  // slots of 128 words (8 MB)

typedef unsigned long long mail_t;
constexpr size_t SR_MAIL_WORDS = size_t(SR_MAIL_SLOTS) * 128;
static __device__ __align__(256) mail_t g_mail[SR_MAIL_WORDS];

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
// Eq. 6 as one fused multiply-add per value: a = 1 / den, b = -min / den - 1/2
__device__ __forceinline__ void coef_from_word(uint32_t w, float& a, float& b) {
    const float mn = bf16lo(w), mx = bf16hi(w);
    float den = mx - mn;
    den = den == 0.0f ? 1.0f : den;
    a = 1.0f / den;
    b = __builtin_fmaf(-mn, a, -0.5f);
}

// ---- sums over the 16 lanes of a row, 16 at a time ---------------------------------------------------------------
// Every lane of a row of 16 holds 16 partial sums p[0 .. 15]; afterwards lane o holds the total of p[o] over the 16
// lanes.  Four exchange steps that halve the number of sums a lane still carries (8 + 4 + 2 + 1 additions per lane
// instead of 16 x 4 for sixteen separate reductions).  Steps over 8 and 4 lanes: one data-parallel addition per
// result, written only by the lanes (banks of four) that keep that result; steps over 2 and 1: a select per operand.
__device__ __forceinline__ void lanes16_step8(const float (&in)[16], float (&out)[8]) {
    // lanes 0-7: out[j] = in[j] + in[j] of lane + 8;  lanes 8-15: out[j] = in[8 + j] + in[8 + j] of lane - 8
    asm("s_nop 1\n\t"
        "v_add_f32_dpp %0, %8, %8 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %1, %9, %9 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %2, %10, %10 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %3, %11, %11 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %4, %12, %12 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %5, %13, %13 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %6, %14, %14 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %7, %15, %15 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %0, %16, %16 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %1, %17, %17 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %2, %18, %18 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %3, %19, %19 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %4, %20, %20 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %5, %21, %21 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %6, %22, %22 row_ror:8 row_mask:0xf bank_mask:0xc\n\t"
        "v_add_f32_dpp %7, %23, %23 row_ror:8 row_mask:0xf bank_mask:0xc"
        : "=&v"(out[0]), "=&v"(out[1]), "=&v"(out[2]), "=&v"(out[3]), "=&v"(out[4]), "=&v"(out[5]), "=&v"(out[6]), "=&v"(out[7])
        : "v"(in[0]), "v"(in[1]), "v"(in[2]), "v"(in[3]), "v"(in[4]), "v"(in[5]), "v"(in[6]), "v"(in[7]),
          "v"(in[8]), "v"(in[9]), "v"(in[10]), "v"(in[11]), "v"(in[12]), "v"(in[13]), "v"(in[14]), "v"(in[15]));
}
__device__ __forceinline__ void lanes16_step4(const float (&in)[8], float (&out)[4]) {
    // lanes with bit 2 clear: out[j] = in[j] + in[j] of lane + 4;  set: out[j] = in[4 + j] + in[4 + j] of lane - 4
    // (row_ror:n hands lane i the value of lane (i - n) mod 16)
    asm("s_nop 1\n\t"
        "v_add_f32_dpp %0, %4, %4 row_ror:12 row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %1, %5, %5 row_ror:12 row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %2, %6, %6 row_ror:12 row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %3, %7, %7 row_ror:12 row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %0, %8, %8 row_ror:4 row_mask:0xf bank_mask:0xa\n\t"
        "v_add_f32_dpp %1, %9, %9 row_ror:4 row_mask:0xf bank_mask:0xa\n\t"
        "v_add_f32_dpp %2, %10, %10 row_ror:4 row_mask:0xf bank_mask:0xa\n\t"
        "v_add_f32_dpp %3, %11, %11 row_ror:4 row_mask:0xf bank_mask:0xa"
        : "=&v"(out[0]), "=&v"(out[1]), "=&v"(out[2]), "=&v"(out[3])
        : "v"(in[0]), "v"(in[1]), "v"(in[2]), "v"(in[3]), "v"(in[4]), "v"(in[5]), "v"(in[6]), "v"(in[7]));
}
__device__ __forceinline__ float quad_swap2(float v) {   // value of lane ^ 2
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4e, 0xf, 0xf, false));
}
__device__ __forceinline__ float quad_swap1(float v) {   // value of lane ^ 1
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xb1, 0xf, 0xf, false));
}
__device__ __forceinline__ float lanes16_transpose_sum(const float (&p)[16], int o) {
    float q8[8], q4[4];
    lanes16_step8(p, q8);
    lanes16_step4(q8, q4);
    const bool b1 = (o & 2) != 0, b0 = (o & 1) != 0;
    const float t0 = (b1 ? q4[2] : q4[0]) + quad_swap2(b1 ? q4[0] : q4[2]);
    const float t1 = (b1 ? q4[3] : q4[1]) + quad_swap2(b1 ? q4[1] : q4[3]);
    return (b0 ? t1 : t0) + quad_swap1(b0 ? t0 : t1);
}

struct ResidentPlan {
    int use;        // the kernel applies
    int nstreams;   // B * Hkv * 2
    int NT;         // threads (= rows) per workgroup: 64, 128 or 256
    int W;          // parts per chunk
    int wgs;        // nstreams * (Ns + 1) * W
};

template <int NT>
struct ResidentLds {
    uint32_t red[NT / 64][16][8];   // per wave and 16-byte column: 4 words of packed min, 4 of packed max
    float coef_a[128], coef_b[128];
    float stage[NT];
    int ready;
};

// 16 bytes at `base + off`: `base` is the same in every lane and stays in scalar registers, the lanes bring 32-bit
// offsets (the addressing form that needs no 64-bit address arithmetic per lane)
typedef __attribute__((address_space(1))) const unsigned char* global_bytes;
__device__ __forceinline__ uint4 load16_scalar_base(const unsigned char* base, unsigned off) {
    global_bytes g = (global_bytes)base;
    asm("" : "+s"(g));
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    // streaming hint: the rows are used once here (measured: 6.8 against 5.8 TB/s for plain loads of this pattern)
    const u32x4 q = __builtin_nontemporal_load(reinterpret_cast<__attribute__((address_space(1))) const u32x4*>(g + off));
    return make_uint4(q.x, q.y, q.z, q.w);
}

__device__ __forceinline__ mail_t mail_load(const mail_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int NT>
__global__ __launch_bounds__(NT) void k_score_resident(Dims D, const bf16_t* __restrict__ Kp, const bf16_t* __restrict__ Vp,
                                                       float* __restrict__ sigma, mail_t* mail, int W, uint32_t tagbase, int spin) {
    constexpr int NW = NT / 64, RS = NT / 16;     // waves; rows per row set (row r + RS * k is piece k of a thread)
    constexpr int PW = NW > 1 ? 1 : 0;            // the wave that polls (wave 0 publishes)
    __shared__ ResidentLds<NT> sh;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nstreams = D.B * D.Hkv * 2;
    const int part = blockIdx.x % W, t = blockIdx.x / W;
    const int s = t % nstreams, c = D.Ns - t / nstreams;           // chunk Ns (reference only) comes first
    const int z = s & 1, bh = s >> 1, b = bh / D.Hkv, h = bh % D.Hkv;
    const bf16_t* Z = (z ? Vp : Kp) + b * D.ks[0] + h * D.ks[1];
    const int r_begin = min(part * NT, D.L - NT);                  // L >= NT
    const int r = tid >> 4, o = tid & 15;
    // first row of the part (the same for the whole workgroup) and this thread's byte offset from it
    const unsigned char* ubase = reinterpret_cast<const unsigned char*>(Z + (int64_t(D.S) + int64_t(c) * D.L + r_begin) * D.ks[2]);
    const unsigned row_bytes = unsigned(D.ks[2]) * 2u;             // < 2^24
    const unsigned voff = unsigned(r) * row_bytes + unsigned(o) * 16u;
    const float inv_d = 1.0f / 128.0f, inv_dof = 1.0f / float(128 - D.ddof);

    uint4 v[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = load16_scalar_base(ubase + size_t(k) * RS * row_bytes, voff);

    auto reduce_to_lds = [&](MinMax8& m) {       // the four rows of a wave (lanes 16, 32 apart), then one record per wave
#pragma unroll
        for (int off = 16; off < 64; off <<= 1) {
            uint32_t omn[4], omx[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) { omn[k] = __shfl_xor(m.mn[k], off, 64); omx[k] = __shfl_xor(m.mx[k], off, 64); }
            m.merge(omn, omx);
        }
        if (lane < 16) {
#pragma unroll
            for (int k = 0; k < 4; ++k) { sh.red[wave][o][k] = m.mn[k]; sh.red[wave][o][4 + k] = m.mx[k]; }
        }
    };
    auto combined_words = [&](uint32_t& w0, uint32_t& w1) {   // channels 2 * lane, 2 * lane + 1: max16 << 16 | min16
        const int col = lane >> 2, wd = lane & 3;
        uint32_t mn = PK_POS_INF, mx = PK_NEG_INF;
#pragma unroll
        for (int wv = 0; wv < NW; ++wv) {
            mn = pk_min(mn, sh.red[wv][col][wd]);
            mx = pk_max(mx, sh.red[wv][col][4 + wd]);
        }
        w0 = ((mx & 0xffffu) << 16) | (mn & 0xffffu);
        w1 = (mx & 0xffff0000u) | (mn >> 16);
    };

    if (c >= 1) {                                  // the min / max of chunk 0 serve nobody
        MinMax8 m;
        m.reset();
#pragma unroll
        for (int k = 0; k < 16; ++k) m.take(v[k]);
        reduce_to_lds(m);
        __syncthreads();
        if (wave == 0) {
            uint32_t w0, w1;
            combined_words(w0, w1);
            const uint32_t tag = tagbase | uint32_t(c);
            mail_t* dst = mail + size_t(blockIdx.x % SR_MAIL_SLOTS) * 128 + 2 * lane;
            mail_store(dst, (mail_t(tag) << 32) | w0);
            mail_store(dst + 1, (mail_t(tag) << 32) | w1);
        }
        if (c == D.Ns) return;                     // reference only
    }

    if (wave == PW) {                              // the words of every part of chunk c + 1
        const uint32_t tag = tagbase | uint32_t(c + 1);
        const unsigned first = (unsigned(D.Ns - (c + 1)) * nstreams + s) * W;   // grid index of part 0 of (s, c + 1)
        float mn0 = INFINITY, mx0 = -INFINITY, mn1 = INFINITY, mx1 = -INFINITY;
        unsigned have = 0;
        const unsigned all = (1u << W) - 1u;
        for (int tries = 0; have != all && tries < spin; ++tries) {
            for (int k0 = 0; k0 < W; k0 += 4) {
                mail_t q[4][2];
#pragma unroll
                for (int i = 0; i < 4; ++i) {      // four parts per round trip; parts past the last repeat it
                    const mail_t* pz = mail + size_t((first + min(k0 + i, W - 1)) % SR_MAIL_SLOTS) * 128 + 2 * lane;
                    q[i][0] = mail_load(pz);
                    q[i][1] = mail_load(pz + 1);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int k = min(k0 + i, W - 1);
                    const bool ok = uint32_t(q[i][0] >> 32) == tag && uint32_t(q[i][1] >> 32) == tag;
                    if ((have >> k & 1u) || __builtin_amdgcn_ballot_w64(!ok) != 0) continue;
                    mn0 = fminf(mn0, bf16lo(uint32_t(q[i][0]))); mx0 = fmaxf(mx0, bf16hi(uint32_t(q[i][0])));
                    mn1 = fminf(mn1, bf16lo(uint32_t(q[i][1]))); mx1 = fmaxf(mx1, bf16hi(uint32_t(q[i][1])));
                    have |= 1u << k;
                }
            }
            if (have != all) __builtin_amdgcn_s_sleep(8);
        }
        if (have == all) {
            float a0, b0, a1, b1;
            coef_from_word((__float_as_uint(mx0) & 0xffff0000u) | (__float_as_uint(mn0) >> 16), a0, b0);
            coef_from_word((__float_as_uint(mx1) & 0xffff0000u) | (__float_as_uint(mn1) >> 16), a1, b1);
            sh.coef_a[2 * lane] = a0; sh.coef_b[2 * lane] = b0;
            sh.coef_a[2 * lane + 1] = a1; sh.coef_b[2 * lane + 1] = b1;
        }
        if (lane == 0) sh.ready = have == all ? 1 : 0;
    }
    __syncthreads();
    if (!sh.ready) {
        // The mailboxes did not deliver: min / max of chunk c + 1 from its rows (every thread: one 16-byte column,
        // rows tid / 16, + RS, ...).  The records in sh.red are free: wave 0 has read them before the barrier above.
        MinMax8 f;
        f.reset();
        const int64_t row0 = int64_t(D.S) + int64_t(c + 1) * D.L;
        for (int rr = r; rr < D.L; rr += RS) f.take(*reinterpret_cast<const uint4*>(Z + (row0 + rr) * D.ks[2] + o * 8));
        reduce_to_lds(f);
        __syncthreads();
        if (wave == 0) {
            uint32_t w0, w1;
            combined_words(w0, w1);
            float a0, b0, a1, b1;
            coef_from_word(w0, a0, b0);
            coef_from_word(w1, a1, b1);
            sh.coef_a[2 * lane] = a0; sh.coef_b[2 * lane] = b0;
            sh.coef_a[2 * lane + 1] = a1; sh.coef_b[2 * lane + 1] = b1;
        }
        __syncthreads();
    }

    float a[8], bq[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = sh.coef_a[8 * o + e]; bq[e] = sh.coef_b[8 * o + e]; }
    // Eq. 6 on this lane's 8 channels of a row
    auto normalise = [&](const uint4& q, float (&x)[8]) {
        const uint32_t wsrc[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            x[2 * k] = __builtin_fmaf(bf16lo(wsrc[k]), a[2 * k], bq[2 * k]);
            x[2 * k + 1] = __builtin_fmaf(bf16hi(wsrc[k]), a[2 * k + 1], bq[2 * k + 1]);
        }
    };
    // Eq. 7, the standard deviation over the 128 channels: this lane's sums over its 8 channels of each of its 16
    // rows, then one exchange that leaves lane o with the totals of row r + RS * o
    float p1[16], p2[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        float x[8];
        normalise(v[k], x);
        float s1 = x[0] + x[1], s2 = x[0] * x[0];
        s2 = __builtin_fmaf(x[1], x[1], s2);
#pragma unroll
        for (int e = 2; e < 8; ++e) {
            s1 += x[e];
            s2 = __builtin_fmaf(x[e], x[e], s2);
        }
        p1[k] = s1;
        p2[k] = s2;
    }
    const float s1 = lanes16_transpose_sum(p1, o), s2 = lanes16_transpose_sum(p2, o);
    const float m2 = s1 * s1 * inv_d;
    float var = s2 - m2;
    const bool cancels = m2 > 0.25f * s2;          // the two terms cancel in the row of this lane
    if (__builtin_amdgcn_ballot_w64(cancels) != 0) {
        // Rare.  The variance of such a row is taken from the deviations about its mean; every lane of the wave
        // goes along, a row that does not need it keeps the value it has.
        const float mean_o = s1 * inv_d;           // of row r + RS * o
        float pq[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            // the mean of row r + RS * k sits in lane k of this row of 16 lanes; the row itself is read again
            const float mean = __shfl(mean_o, (lane & 48) | k, 64);
            const uint4 q = load16_scalar_base(ubase + size_t(k) * RS * row_bytes, voff);
            float x[8];
            normalise(q, x);
            float qd = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) { const float dv = x[e] - mean; qd = __builtin_fmaf(dv, dv, qd); }
            pq[k] = qd;
        }
        const float var2 = lanes16_transpose_sum(pq, o);
        var = cancels ? var2 : var;
    }
    sh.stage[r + RS * o] = __builtin_amdgcn_sqrtf(fmaxf(var, 0.0f) * inv_dof);
    __syncthreads();
    sigma[(int64_t(s) * D.Ns + c) * D.L + r_begin + tid] = sh.stage[tid];
}

static ResidentPlan make_resident_plan(const Dims& D) {
    ResidentPlan P = {};
    P.nstreams = D.B * D.Hkv * 2;
    P.NT = D.L >= 256 ? 256 : D.L >= 128 ? 128 : 64;
    P.W = (D.L + P.NT - 1) / P.NT;
    const int64_t wgs = int64_t(P.nstreams) * (D.Ns + 1) * P.W;
    P.wgs = int(wgs);
    // slots: a reader's writers are at most nstreams * W + W workgroups before it, and a writer's words must outlive
    // every workgroup that may still be running when it is dispatched (a quarter of the slots and more)
    P.use = D.dtype == 1 && D.d == 128 && D.Ns > 0 && D.Ns + 1 <= SR_MAX_CHUNKS && D.L >= 64 && D.ks[2] % 8 == 0 &&
            D.ks[2] <= (int64_t(1) << 22) && P.W <= SR_MAX_PARTS && int64_t(P.nstreams) * P.W * 2 <= SR_MAIL_SLOTS / 2 &&
            wgs <= (int64_t(1) << 30);
    return P;
}

// Softmax over the chunk's tokens for K and V, summed (Eq. 7-8); SELECT: the chunk's top K right away (text after
// Eq. 8).  One workgroup of NT threads per (batch, KV head, chunk).  The work is a chain of short block-wide
// reductions and scans: with many chunks small workgroups (several per CU) finish soonest, with few chunks (fewer
// than CUs) the chain itself is the time and more threads shorten it.  A thread keeps its rows in registers from the
// load to the score; dynamic LDS: L floats (the scores, for the selection).  The workgroups also clear the mailbox
// words that the scoring kernel of this call may have written.
template <bool SELECT, int NT>
__global__ __launch_bounds__(NT) void k_softmax_select(Dims D, const float* __restrict__ sigma, float* __restrict__ score,
                                                       int32_t* __restrict__ idx, mail_t* mail, int mail_words) {
    constexpr int NW = NT / 64, MAXJ = FUSED_MAX_L / NT;   // rows tid, tid + NT, ... of a thread: at most MAXJ
    const int p = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    extern __shared__ float sx_key[];     // [L]: the scores, for the selection
    __shared__ float sm[2 * NW];
    // the mailbox words first: the stores drain while the standard deviations are on their way
    const int64_t g = int64_t(bh) * gridDim.x + p, G = int64_t(gridDim.x) * gridDim.y;
    for (int64_t e = g * NT + tid; e < mail_words; e += G * NT) mail[e] = 0;
    const float* sk = sigma + ((int64_t(bh) * 2 + 0) * D.Ns + p) * D.L;
    const float* sv = sigma + ((int64_t(bh) * 2 + 1) * D.Ns + p) * D.L;
    // The thread's rows stay in registers; a row past the chunk counts as -inf (its exponential is 0).
    float vk[MAXJ], vv[MAXJ];
#pragma unroll
    for (int j = 0; j < MAXJ; ++j) {
        const int r = tid + j * NT;
        const bool in = j * NT < D.L && r < D.L;
        vk[j] = in ? sk[r] : -INFINITY;
        vv[j] = in ? sv[r] : -INFINITY;
    }
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
#pragma unroll
    for (int j = 0; j < MAXJ; ++j) { mk = fmaxf(mk, vk[j]); mv = fmaxf(mv, vv[j]); }
    block_red2(mk, mv, true);
    float zk = 0.0f, zv = 0.0f;
#pragma unroll
    for (int j = 0; j < MAXJ; ++j) {
        if (j * NT < D.L) {
            vk[j] = expf(vk[j] - mk);
            vv[j] = expf(vv[j] - mv);
            zk += vk[j];
            zv += vv[j];
        }
    }
    block_red2(zk, zv, false);
    float* out = score + (int64_t(bh) * D.Ns + p) * D.L;
#pragma unroll
    for (int j = 0; j < MAXJ; ++j) {
        const int r = tid + j * NT;
        if (j * NT < D.L && r < D.L) {
            const float sc = vk[j] / zk + vv[j] / zv;      // Eq. 7-8
            out[r] = sc;
            if (SELECT) sx_key[r] = sc;
        }
    }
    if (SELECT) {
        __shared__ SelectLds sel;
        __syncthreads();
        select_topk_block<NT>(reinterpret_cast<const uint32_t*>(sx_key), D.L, D.K, D.S + p * D.L,
                              idx + (int64_t(bh) * D.Ns + p) * D.K, sel);
    }
}

static hipError_t run_softmax_select(const Dims& D, const float* sigma, float* score, int32_t* idx, mail_t* mail,
                                     int mail_words, hipStream_t st) {
    const size_t lds = size_t(D.L) * sizeof(float);
    const dim3 grid(D.Ns, D.B * D.Hkv);
    // threads per chunk (measured): chunks of 1024 rows and more take 1024 threads when there are at most half as many
    // chunks as CUs and 512 when at most two per CU (C4: 12.4 -> 11.3 us, C5: 22.9 -> 18.9 us against 256 threads);
    // shorter or more chunks take 256 (C3, 992 chunks of 512 rows: 13.3 us against 15.7 us with 512)
    const int64_t chunks = int64_t(D.Ns) * D.B * D.Hkv;
    const int nt = D.L >= 1024 && chunks <= 128 ? 1024 : D.L >= 1024 && chunks <= 512 ? 512 : 256;
#define LRSA_SX(name, SEL, NT_) \
    LRSA_TIMED_LAUNCH(name, st, (k_softmax_select<SEL, NT_>), grid, dim3(NT_), lds, st, D, sigma, score, idx, mail, mail_words)
    if (idx) {
        if (nt == 1024) LRSA_SX("k_softmax_select", true, 1024);
        else if (nt == 512) LRSA_SX("k_softmax_select", true, 512);
        else LRSA_SX("k_softmax_select", true, 256);
    } else {
        if (nt == 1024) LRSA_SX("k_softmax", false, 1024);
        else if (nt == 512) LRSA_SX("k_softmax", false, 512);
        else LRSA_SX("k_softmax", false, 256);
    }
#undef LRSA_SX
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ host side
namespace {
struct DeviceState {
    mail_t* mail = nullptr;
};
std::mutex g_mu;
DeviceState g_dev[64];
std::atomic<uint32_t> g_seq{0};
std::atomic<int> g_spin{SR_SPIN};

// address of the mailboxes on the current device, looked up once per device
hipError_t device_state(DeviceState* out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_mu);
    DeviceState& st = g_dev[dev];
    if (!st.mail) {
        void* pp = nullptr;
        if ((e = hipGetSymbolAddress(&pp, HIP_SYMBOL(g_mail))) != hipSuccess) return e;
        if (!pp) return hipErrorInvalidSymbol;
        st.mail = static_cast<mail_t*>(pp);
    }
    *out = st;
    return hipSuccess;
}
}  // namespace

// Eq. 7-8 (and the selection when idx is given) from standard deviations that other kernels left in `sigma`
hipError_t launch_softmax_select(const Dims& D, const float* sigma, float* score, int32_t* idx, hipStream_t st) {
    return run_softmax_select(D, sigma, score, idx, nullptr, 0, st);
}

bool score_resident_applies(const Dims& D) { return make_resident_plan(D).use != 0; }

int score_poll_limit(int polls) {
    return polls < 0 ? g_spin.load() : g_spin.exchange(polls > (1 << 20) ? (1 << 20) : polls);
}

// scores (and, with idx, the selection) through the chunk-resident kernel; sigma: B * Hkv * 2 * Ns * L floats of workspace
hipError_t launch_score_resident(const Dims& D, const void* K, const void* V, float* score, int32_t* idx, float* sigma,
                                 hipStream_t st) {
    DeviceState ds;
    const hipError_t e = device_state(&ds);
    if (e != hipSuccess) return e;
    const ResidentPlan P = make_resident_plan(D);
    const uint32_t seq = g_seq.fetch_add(1) % 0xfffffu + 1u;          // 1 .. 2^20 - 1: a tag is never zero
    const int spin = g_spin.load();
#define LRSA_SR(NT_) \
    LRSA_TIMED_LAUNCH("k_score_resident", st, (k_score_resident<NT_>), dim3(P.wgs), dim3(NT_), 0, st, D, (const bf16_t*)K, \
                      (const bf16_t*)V, sigma, ds.mail, P.W, seq << 12, spin)
    if (P.NT == 256) LRSA_SR(256); else if (P.NT == 128) LRSA_SR(128); else LRSA_SR(64);
#undef LRSA_SR
    return run_softmax_select(D, sigma, score, idx, ds.mail, (P.wgs < SR_MAIL_SLOTS ? P.wgs : SR_MAIL_SLOTS) * 128, st);
}

}  // namespace lrsa
