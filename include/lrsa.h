/* lrsa.h -- C ABI of the MI355X (gfx950) hot path of Lag-Relative Sparse Attention (LRSA).
 *
 * The path, in the paper's notation (Method section): per attention head i the states
 * Q_i, K_i, V_i in R^{n x d_h} (Eq. 1); the KV sequence is split into a sink of S tokens and
 * chunks of the lag size L; each chunk p is scored against the chunk after it (Eq. 4-8); the
 * top r*L = K tokens of every chunk survive (text after Eq. 8); attention (Eq. 2-3) runs under
 * the chunked mask of the "Attention Filling" steps: a query sees the sink, the survivors of
 * every chunk that lies more than `local_prev` chunks behind its own, the `local_prev` chunks
 * before its own in full, and its own chunk causally.
 *
 * Conventions for every call
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library neither frees
 *     nor keeps them after the call returns.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream);
 *     the call returns without synchronising.
 *   - `ws` is a caller-owned device scratch buffer of at least lrsa_workspace_bytes() bytes,
 *     256-byte aligned; it may be NULL when that size is 0.  Its contents are undefined after
 *     the call.  Calls that share one workspace must be ordered on one stream.
 *   - Outputs are fully overwritten; they need not be initialised.
 *   - Return value: LRSA_OK (0) or a negative lrsa_status.  Arguments are validated before
 *     any HIP call, so argument errors are reported without touching the GPU.  The library
 *     never aborts and throws nothing.  lrsa_last_error() describes the last failure of the
 *     calling thread.
 *   - NaN/Inf in the inputs give undefined results and are not checked.
 *
 * Partition (text after Eq. 8): P = floor((n-S)/L) full chunks C_p = [S+pL, S+(p+1)L), a tail
 * of R = n-S-PL tokens that forms one more query chunk, nq = P + (R>0) query chunks, and
 * Ns = max(nq-1-local_prev, 0) chunks that are ever seen compressed and therefore scored.
 */
#ifndef LRSA_H
#define LRSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LRSA_OK = 0,
    LRSA_ERR_INVALID_ARG = -1, /* null pointer, K > L, heads_q % heads_kv != 0, bad stride, small ws ... */
    LRSA_ERR_UNSUPPORTED = -2, /* head_dim / dtype combination that is not built                         */
    LRSA_ERR_HIP = -3          /* a HIP call failed; the message carries hipGetErrorString                */
} lrsa_status;

typedef enum { LRSA_F32 = 0, LRSA_BF16 = 1 } lrsa_dtype;

/* Which kernels serve the attention calls. */
typedef enum {
    LRSA_IMPL_AUTO = 0,    /* bf16 with head_dim 128: MFMA kernels; everything else: generic kernels */
    LRSA_IMPL_GENERIC = 1, /* force the plain fp32-arithmetic kernels (any supported dtype/head_dim)  */
    LRSA_IMPL_COMPACT = 2  /* MFMA kernels over a physically condensed KV cache: lrsa_attn_fwd and
                              lrsa_attn_bwd first copy the rows of the gather list (sink, survivors) into
                              a contiguous buffer in the workspace and read that instead of gathering by
                              index in their loops; same results bit for bit, a larger workspace.  Where
                              the MFMA kernels do not apply it behaves like LRSA_IMPL_AUTO.            */
} lrsa_impl;

typedef struct {
    int32_t batch;         /* B >= 1                                                                 */
    int32_t heads_q;       /* query heads; heads_q % heads_kv == 0, group size G = heads_q/heads_kv  */
    int32_t heads_kv;      /* KV heads; scores and the selection are per KV head                     */
    int32_t seq;           /* n >= 1                                                                 */
    int32_t head_dim;      /* d_h: 64 or 128                                                         */
    int32_t sink;          /* S >= 0                                                                 */
    int32_t lag;           /* L >= 2: lag = chunk size                                               */
    int32_t topk;          /* K = r*L survivors per chunk, 1 <= K <= L                               */
    int32_t std_ddof;      /* divisor of Std in Eq. 7 is d_h - std_ddof; 0 or 1 (the paper is silent, 1 is the default reading) */
    int32_t local_prev;    /* chunks kept in full before the query's own chunk, >= 1; 1 is the paper's sliding window */
    float softmax_scale;   /* <= 0 selects 1/sqrt(d_h) of Eq. 3                                      */
    int32_t dtype;         /* lrsa_dtype of Q, K, V, O, dO, dQ, dK, dV                               */
    int32_t impl;          /* lrsa_impl                                                              */
    int64_t q_stride[3];   /* element strides of (batch, head, position) for Q, O, dO, dQ            */
    int64_t kv_stride[3];  /* element strides of (batch, head, position) for K, V, dK, dV            */
                           /* the channel stride is 1; position stride >= head_dim; rows 16-byte aligned */
} lrsa_params;

/* Which call a workspace size is asked for. */
typedef enum {
    LRSA_WS_SCORE = 0, LRSA_WS_SELECT = 1, LRSA_WS_ATTN_FWD = 2, LRSA_WS_ATTN_BWD = 3,
    LRSA_WS_DECODE_ATTN = 4 /* lrsa_decode_attn; lrsa_cache_compress needs none */
} lrsa_ws_kind;

/* Ns of the partition above; pure host arithmetic.  Returns a negative lrsa_status on bad params. */
int lrsa_num_scored_chunks(const lrsa_params *p);

/* Which kernels lrsa_score / lrsa_score_select use for these params (Eq. 4-8 are the same on every route, the
 * routes differ in how the rows are spread over the chip); pure host arithmetic, for tests and for reading
 * profiles.  0: nothing to score (Ns == 0); 1: one workgroup per (batch, KV head, chunk); 2: chunks cut into
 * row slices, three launches (few, long chunks); 3: the one-read kernel, which keeps the rows in registers
 * from their min / max to their scores (bf16, head_dim 128, chunks of 64 to 4096 rows); 4: chunks beyond
 * 4096 tokens.  Returns a negative lrsa_status on bad params. */
int lrsa_score_route(const lrsa_params *p);

/* On route 3 a scoring workgroup takes the min / max of its reference chunk (Eq. 4-5) from hint words that
 * the workgroups of that chunk publish; `polls` is how many times it looks for them before it computes
 * these min / max from the rows themselves (a second read of the chunk).  Default 256 (about a
 * millisecond); 0: never wait (every chunk is read twice).  Scores and selections are the same bits for
 * every value: the setting trades time only.  Process-wide, takes effect with the next call; negative:
 * change nothing.  Returns the previous value. */
int lrsa_score_poll_limit(int polls);

/* Bytes of device scratch the call `which` (lrsa_ws_kind) needs for these params; host arithmetic.
 * Returns 0 for bad params (the call itself then reports the error). */
size_t lrsa_workspace_bytes(const lrsa_params *p, int which);

/* LagKV score, Eq. 4-8.  For Z in {K, V}, every (b, KV head h, chunk p < Ns): per-channel min and
 * max over the rows of chunk p+1 (Eq. 4-5); rows of chunk p normalised with them (Eq. 6; a channel
 * with max == min is divided by 1); Std over the d_h channels of each row, then Softmax over the L
 * rows of the chunk (Eq. 7); score = score(K) + score(V) (Eq. 8).  fp32 arithmetic on the stored
 * values.
 *   K, V  : [B, Hkv, n, d_h] by kv_stride, dtype `dtype`                       (device, read)
 *   score : [B, Hkv, Ns, L] fp32, contiguous                                    (device, written)
 * Ns == 0 is legal: nothing is written and score may be NULL. */
int lrsa_score(const lrsa_params *p, const void *K, const void *V, float *score,
               void *ws, size_t ws_bytes, void *stream);

/* Top-K per head and lag window (text after Eq. 8): for every (b, h, p) the K positions of chunk p
 * with the largest score; equal scores go to the lowest position.
 *   score : [B, Hkv, Ns, L] fp32, contiguous, every value > 0                   (device, read)
 *   idx   : [B, Hkv, Ns, K] int32, contiguous; absolute positions in
 *           [S+pL, S+(p+1)L), strictly ascending                                (device, written)
 * Ns == 0 is legal: nothing is written and both pointers may be NULL. */
int lrsa_select(const lrsa_params *p, const float *score, int32_t *idx,
                void *ws, size_t ws_bytes, void *stream);

/* lrsa_score followed by lrsa_select in one call: the kernel that finishes the scores of a chunk
 * (Eq. 4-8) takes its top K while they are still in LDS (text after Eq. 8), so no selection launch
 * and no second read of the scores is needed (one to three launches, depending on the shape).  Writes
 * exactly what the two calls would write: score and idx are bit-identical to theirs.  Arguments as in
 * lrsa_score and lrsa_select; the workspace is the one of lrsa_score (LRSA_WS_SCORE).  Ns == 0 is
 * legal: nothing is written.
 * On route 3 (lrsa_score_route; lrsa_score takes it too) the scoring kernel keeps small hint words in 8 MB
 * of device memory that the library owns; calls that score on the same GPU at the same time (different
 * streams or threads) may overwrite each other's hints, which costs time, never results. */
int lrsa_score_select(const lrsa_params *p, const void *K, const void *V, float *score, int32_t *idx,
                      void *ws, size_t ws_bytes, void *stream);

/* Debug aid for callers that bring their own idx (text after Eq. 8 fixes what a valid selection is): counts
 * the rows (b, h, p) of idx that break the precondition of the attention calls -- K positions inside chunk p,
 * [S+pL, S+(p+1)L), strictly ascending -- which those calls do not check.
 *   idx      : [B, Hkv, Ns, K] int32, contiguous; may be NULL when Ns == 0          (device, read)
 *   bad_rows : one int32; receives the number of offending rows, 0 for a valid idx   (device, written)
 * Enqueued on `stream` like every call; read bad_rows after synchronising. */
int lrsa_check_idx(const lrsa_params *p, const int32_t *idx, int32_t *bad_rows, void *stream);

/* Attention forward, Eq. 2-3 under the chunked mask: O[t] = sum_u softmax_u(scale q_t.k_u) v_u over
 * the keys u <= t that are in the sink, in the local window of t's chunk, or listed in idx;
 * lse[t] = log sum_u exp(scale q_t.k_u).  Query head hq reads KV head hq / G.
 *   Q     : [B, Hq, n, d_h] by q_stride; K, V: [B, Hkv, n, d_h] by kv_stride    (device, read)
 *   idx   : [B, Hkv, Ns, K] int32 as written by lrsa_select; may be NULL when Ns == 0.
 *           PRECONDITION (not checked on the device): row p holds K distinct positions of chunk p,
 *           [S+pL, S+(p+1)L), strictly ascending.  Positions outside the sequence are read out of
 *           bounds; a row that is not ascending sends gradients to wrong rows of dK, dV.
 *                                                                                (device, read)
 *   O     : [B, Hq, n, d_h] by q_stride, dtype `dtype`                           (device, written)
 *   lse   : [B, Hq, n] fp32, contiguous                                          (device, written)
 * idx is an input, so any valid selection (for instance one computed elsewhere) can be used. */
int lrsa_attn_fwd(const lrsa_params *p, const void *Q, const void *K, const void *V, const int32_t *idx,
                  void *O, float *lse, void *ws, size_t ws_bytes, void *stream);

/* Attention backward: gradients of sum(O * dO) with the mask held constant (the selection carries
 * no gradient).  With A = exp(scale Q K^T + M - lse): dV = A^T dO, dA = dO V^T,
 * D = rowsum(dO * O), dS = A * (dA - D), dQ = scale dS K, dK = scale dS^T Q; dK and dV are summed
 * over the G query heads of a group.
 *   Q, K, V, idx as in lrsa_attn_fwd; O, lse as written by it; dO like O        (device, read)
 *   dQ    : like Q; dK, dV: like K                                               (device, written)
 */
int lrsa_attn_bwd(const lrsa_params *p, const void *Q, const void *K, const void *V, const void *O,
                  const void *dO, const float *lse, const int32_t *idx,
                  void *dQ, void *dK, void *dV, void *ws, size_t ws_bytes, void *stream);

/* ---- attention by filling steps (Section 3.2, "Attention Filling 1 / 2 / repeat": the sequence is attended a few
 * chunks at a time against a cache of sink + survivors + the previous chunk, so that the activations that live at
 * once are those of m chunks, not of the whole sequence).
 *
 * A step covers the query rows [row_begin, row_end): row_begin is 0 or a chunk start S + qL, row_end a chunk start
 * or the end of the sequence; the sink rows belong to the step that starts at 0.  The mask is the one of
 * lrsa_attn_fwd (it does not depend on how many chunks a step takes), so the steps together give exactly the
 * results of the one-shot calls: O, lse and dQ bit for bit, dK and dV up to the order of fp32 additions.
 *   Q, O, dO, dQ : [B, Hq, row_end - row_begin, d_h] by q_stride -- the rows of the step only
 *   lse          : [B, Hq, row_end - row_begin] fp32, contiguous
 *   K, V         : [B, Hkv, n, d_h] by kv_stride; rows at and after row_end are not read
 *   idx          : [B, Hkv, Ns, K] as for lrsa_attn_fwd; only the rows of chunks that are compressed for the step's
 *                  queries (chunks < row_end's chunk - local_prev) are read, later rows may still be unwritten
 *   dK_acc, dV_acc : [B, Hkv, n, d_h] fp32, contiguous: lrsa_attn_bwd_fill ADDS the step's share (the caller zeroes
 *                  them before the first step; steps in any order, one after the other on one stream);
 *                  lrsa_attn_bwd_finish converts the sums to dK, dV (by kv_stride, dtype `dtype`)
 * Workspace: lrsa_fill_workspace_bytes(p, row_begin, row_end, LRSA_WS_ATTN_FWD / LRSA_WS_ATTN_BWD) -- it grows
 * with the rows of the step and the cache they see, not with n * n_q.  Built for bf16 with head_dim 128
 * (LRSA_ERR_UNSUPPORTED otherwise); impl LRSA_IMPL_COMPACT is treated as LRSA_IMPL_AUTO. */
size_t lrsa_fill_workspace_bytes(const lrsa_params *p, int32_t row_begin, int32_t row_end, int which);
int lrsa_attn_fwd_fill(const lrsa_params *p, int32_t row_begin, int32_t row_end, const void *Q, const void *K,
                       const void *V, const int32_t *idx, void *O, float *lse, void *ws, size_t ws_bytes, void *stream);
int lrsa_attn_bwd_fill(const lrsa_params *p, int32_t row_begin, int32_t row_end, const void *Q, const void *K,
                       const void *V, const void *O, const void *dO, const float *lse, const int32_t *idx, void *dQ,
                       float *dK_acc, float *dV_acc, void *ws, size_t ws_bytes, void *stream);
int lrsa_attn_bwd_finish(const lrsa_params *p, const float *dK_acc, const float *dV_acc, void *dK, void *dV,
                         void *stream);

/* ---- inference-time LagKV cache (the setting of the paper's evaluation: the cache compressed lag window by
 * lag window while tokens are generated; Section 3.2, Attention Filling 1: once a second chunk is complete the
 * chunk before it is cut down to its survivors and the newer one stays whole as the local window).
 *
 * Cache of one layer: Kc, Vc [B, Hkv, cap, d_h] by kv_stride with cap = p->seq; rows [0, len) valid, the same
 * len for every head: the sink rows, then topk rows per compressed chunk, then the uncompressed tail.
 * heads_q, sink, lag, topk, std_ddof, dtype as for the other calls; local_prev must be 1; lag <= 4096.
 *
 * lrsa_cache_compress: while the tail holds at least 2*lag rows, the first lag rows of the tail are scored
 * against the next lag rows (Eq. 4-8), their top `topk` rows are kept in position order (text after Eq. 8,
 * ties to the lowest position) and the rest of the tail moves down, in place.  Call it BEFORE appending the
 * next token: a token attends first, the chunk before its own is compressed only when the following token
 * arrives -- the cache is then exactly what the training-time mask lets that token see.
 *   Kc, Vc : device, read and written in place
 *   pos    : [B, Hkv, cap] int32, contiguous, the original position of every row; moved alike; may be NULL
 *   len, done : valid rows and chunks compressed so far (host values)
 *   len_out, done_out : HOST pointers, receive the new values (pure host arithmetic, no synchronisation)
 * Nothing is launched when the tail is shorter than 2*lag. */
int lrsa_cache_compress(const lrsa_params *p, void *Kc, void *Vc, int32_t *pos, int32_t len, int32_t done,
                        int32_t *len_out, int32_t *done_out, void *stream);

/* Single-query attention over the cache (Eq. 3, every cache row visible): for each query head,
 * O = softmax(scale q.Kc^T) Vc over rows [0, len).  Query head hq reads KV head hq / G.
 *   q   : [B, Hq, d_h] contiguous, dtype `dtype`                                  (device, read)
 *   O   : [B, Hq, d_h] contiguous, dtype `dtype`                                  (device, written)
 *   lse : [B, Hq] fp32 log-sum-exp of the scaled logits, may be NULL              (device, written)
 * 1 <= len <= cap.  Workspace: LRSA_WS_DECODE_ATTN. */
int lrsa_decode_attn(const lrsa_params *p, const void *q, const void *Kc, const void *Vc, int32_t len, void *O,
                     float *lse, void *ws, size_t ws_bytes, void *stream);

/* lrsa_decode_attn for callers that cannot allocate device memory or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results (bit
 * for bit) as lrsa_decode_attn, but the partial records of the key slices live in an array inside the library
 * (LRSA_DECODE_STATIC_SCRATCH_BYTES per GPU, held until the process ends) instead of `ws`.  The call allocates
 * and frees nothing (leave lrsa_timing_enable off: timing creates events); the first call on a device looks up
 * the array's address on that device.  A call that needs more than the array holds --
 * batch * heads_q * slices * (head_dim + 2) * 4 bytes, slices = min(256, ceil(len / 256),
 * ceil(512 / (batch * heads_kv))) -- fails with LRSA_ERR_INVALID_ARG and launches nothing.
 * All calls on one GPU share the one array: calls that overlap in time on the same GPU (different streams,
 * different threads) race; order them on one stream.  Nothing needs clearing between calls. */
#define LRSA_DECODE_STATIC_SCRATCH_BYTES (4u << 20)
int lrsa_decode_attn_static(const lrsa_params *p, const void *q, const void *Kc, const void *Vc, int32_t len,
                            void *O, float *lse, void *stream);

/* Message of the calling thread's last failed call (static thread-local storage, never NULL). */
const char *lrsa_last_error(void);

/* Per-kernel timing for benchmarks (not part of the paper's method).  lrsa_timing_enable(1) clears
 * the records and makes every later call bracket each of its kernel launches with HIP events on
 * the call's stream; lrsa_timing_enable(0) clears and stops.  lrsa_timing_count() is the number of
 * launches recorded so far (at most 4096); lrsa_timing_read(i, &name, &ms) waits for launch i and
 * returns its kernel's name (static storage) and duration in milliseconds. */
int lrsa_timing_enable(int on);
int lrsa_timing_count(void);
int lrsa_timing_read(int i, const char **name, float *ms);

/* ABI revision of this header; bumped when a signature or the struct changes. */
int lrsa_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LRSA_H */
