// C-ABI entry points of liblrsa: argument validation (before any HIP call), derived partition,
// and dispatch to the kernel launchers.  Declarations and contracts are in include/lrsa.h.
#include "../../include/lrsa.h"
#include "common.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// Validates the params and fills the derived dimensions.  Touches no HIP API.
int make_dims(const lrsa_params* p, lrsa::Dims* D) {
    if (!p) return fail(LRSA_ERR_INVALID_ARG, "params is NULL");
    if (p->batch < 1 || p->heads_q < 1 || p->heads_kv < 1 || p->seq < 1)
        return fail(LRSA_ERR_INVALID_ARG, "batch, heads_q, heads_kv and seq must be >= 1");
    if (p->heads_q % p->heads_kv != 0)
        return fail(LRSA_ERR_INVALID_ARG, "heads_q (%d) is not a multiple of heads_kv (%d)", p->heads_q, p->heads_kv);
    if (p->sink < 0) return fail(LRSA_ERR_INVALID_ARG, "sink must be >= 0");
    if (p->lag < 2) return fail(LRSA_ERR_INVALID_ARG, "lag must be >= 2");
    if (p->topk < 1 || p->topk > p->lag)
        return fail(LRSA_ERR_INVALID_ARG, "topk (%d) must be in [1, lag=%d]", p->topk, p->lag);
    if (p->std_ddof != 0 && p->std_ddof != 1) return fail(LRSA_ERR_INVALID_ARG, "std_ddof must be 0 or 1");
    if (p->local_prev < 1)
        return fail(LRSA_ERR_INVALID_ARG, "local_prev must be >= 1 (0 would let a query use a selection made from later tokens)");
    if (p->dtype != LRSA_F32 && p->dtype != LRSA_BF16) return fail(LRSA_ERR_UNSUPPORTED, "dtype %d is not built", p->dtype);
    if (p->head_dim != 64 && p->head_dim != 128)
        return fail(LRSA_ERR_UNSUPPORTED, "head_dim %d is not built (64 and 128 are)", p->head_dim);
    if (p->impl != LRSA_IMPL_AUTO && p->impl != LRSA_IMPL_GENERIC && p->impl != LRSA_IMPL_COMPACT)
        return fail(LRSA_ERR_INVALID_ARG, "unknown impl %d", p->impl);
    if (!(p->softmax_scale == p->softmax_scale) || std::isinf(p->softmax_scale))
        return fail(LRSA_ERR_INVALID_ARG, "softmax_scale is not finite");
    const int vec = p->dtype == LRSA_F32 ? 4 : 8;  // elements per 16 bytes
    const int64_t* strides[2] = {p->q_stride, p->kv_stride};
    for (int s = 0; s < 2; ++s) {
        const int64_t* st = strides[s];
        if (st[2] < p->head_dim) return fail(LRSA_ERR_INVALID_ARG, "%s position stride %lld < head_dim", s ? "kv" : "q", (long long)st[2]);
        for (int i = 0; i < 3; ++i) {
            if (st[i] < 0) return fail(LRSA_ERR_INVALID_ARG, "negative stride");
            if (st[i] % vec != 0) return fail(LRSA_ERR_INVALID_ARG, "%s stride %lld breaks 16-byte row alignment", s ? "kv" : "q", (long long)st[i]);
        }
    }
    if ((int64_t)p->seq * p->heads_q > (int64_t)1 << 40) return fail(LRSA_ERR_INVALID_ARG, "problem too large");

    D->B = p->batch; D->Hq = p->heads_q; D->Hkv = p->heads_kv; D->G = p->heads_q / p->heads_kv;
    D->n = p->seq; D->d = p->head_dim; D->S = p->sink; D->L = p->lag; D->K = p->topk;
    D->ddof = p->std_ddof; D->lp = p->local_prev;
    const int64_t rest = p->seq > p->sink ? (int64_t)p->seq - p->sink : 0;
    D->P = (int)(rest / p->lag);
    D->R = (int)(rest - (int64_t)D->P * p->lag);
    D->nq = D->P + (D->R > 0 ? 1 : 0);
    D->Ns = D->nq - 1 - D->lp > 0 ? D->nq - 1 - D->lp : 0;
    D->scale = p->softmax_scale > 0.0f ? p->softmax_scale : 1.0f / std::sqrt((float)p->head_dim);
    D->dtype = p->dtype;
    D->compact = p->impl == LRSA_IMPL_COMPACT ? 1 : 0;
    for (int i = 0; i < 3; ++i) { D->qs[i] = p->q_stride[i]; D->ks[i] = p->kv_stride[i]; }
    D->row_begin = 0; D->row_end = D->n; D->fq0 = 0; D->fq1 = D->nq;      // every query row
    D->lse_stride = D->n;
    D->acc = 0;
    if (p->batch * (int64_t)p->heads_kv * 2 > 65535 || p->heads_q > 65535 || D->Ns > 65535)
        return fail(LRSA_ERR_UNSUPPORTED, "batch*heads or chunk count beyond the launch grid limits");
    return LRSA_OK;
}

bool use_mfma(const lrsa_params* p, const lrsa::Dims& D) { return p->impl != LRSA_IMPL_GENERIC && lrsa::mfma_supported(D); }

size_t ws_need(const lrsa_params* p, const lrsa::Dims& D, int which) {
    switch (which) {
        case LRSA_WS_SCORE: return lrsa::score_ws_bytes(D);
        case LRSA_WS_SELECT: return lrsa::select_ws_bytes(D);
        case LRSA_WS_ATTN_FWD: return use_mfma(p, D) ? lrsa::attn_fwd_mfma_ws_bytes(D) : lrsa::attn_fwd_generic_ws_bytes(D);
        case LRSA_WS_ATTN_BWD: return use_mfma(p, D) ? lrsa::attn_bwd_mfma_ws_bytes(D) : lrsa::attn_bwd_generic_ws_bytes(D);
        case LRSA_WS_DECODE_ATTN: return lrsa::decode_ws_bytes(D);
        default: return 0;
    }
}

int check_ws(const lrsa_params* p, const lrsa::Dims& D, int which, const void* ws, size_t ws_bytes) {
    const size_t need = ws_need(p, D, which);
    if (need == 0) return LRSA_OK;
    if (!ws) return fail(LRSA_ERR_INVALID_ARG, "workspace is NULL but %zu bytes are needed", need);
    if (ws_bytes < need) return fail(LRSA_ERR_INVALID_ARG, "workspace has %zu bytes, %zu are needed", ws_bytes, need);
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return fail(LRSA_ERR_INVALID_ARG, "workspace is not 256-byte aligned");
    return LRSA_OK;
}

int hip_result(hipError_t e, const char* what) {
    if (e == hipSuccess) return LRSA_OK;
    return fail(LRSA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

bool misaligned16(const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 != 0; }

}  // namespace

extern "C" {

int lrsa_abi_version(void) { return 1; }

const char* lrsa_last_error(void) { return g_err; }

int lrsa_num_scored_chunks(const lrsa_params* p) {
    lrsa::Dims D;
    const int rc = make_dims(p, &D);
    return rc != LRSA_OK ? rc : D.Ns;
}

int lrsa_score_route(const lrsa_params* p) {
    lrsa::Dims D;
    const int rc = make_dims(p, &D);
    return rc != LRSA_OK ? rc : lrsa::score_route(D);
}

int lrsa_score_poll_limit(int polls) { return lrsa::score_poll_limit(polls); }

size_t lrsa_workspace_bytes(const lrsa_params* p, int which) {
    lrsa::Dims D;
    if (make_dims(p, &D) != LRSA_OK) return 0;
    return ws_need(p, D, which);
}

int lrsa_score(const lrsa_params* p, const void* K, const void* V, float* score, void* ws, size_t ws_bytes,
               void* stream) {
    lrsa::Dims D;
    int rc = make_dims(p, &D);
    if (rc != LRSA_OK) return rc;
    if (D.Ns == 0) return LRSA_OK;
    if (!K || !V || !score) return fail(LRSA_ERR_INVALID_ARG, "lrsa_score: K, V and score must not be NULL");
    if (misaligned16(K) || misaligned16(V)) return fail(LRSA_ERR_INVALID_ARG, "lrsa_score: K and V must be 16-byte aligned");
    if ((rc = check_ws(p, D, LRSA_WS_SCORE, ws, ws_bytes)) != LRSA_OK) return rc;
    return hip_result(lrsa::launch_score(D, K, V, score, ws, (hipStream_t)stream), "lrsa_score");
}

int lrsa_select(const lrsa_params* p, const float* score, int32_t* idx, void* ws, size_t ws_bytes, void* stream) {
    lrsa::Dims D;
    int rc = make_dims(p, &D);
    if (rc != LRSA_OK) return rc;
    if (D.Ns == 0) return LRSA_OK;
    if (!score || !idx) return fail(LRSA_ERR_INVALID_ARG, "lrsa_select: score and idx must not be NULL");
    if ((rc = check_ws(p, D, LRSA_WS_SELECT, ws, ws_bytes)) != LRSA_OK) return rc;
    return hip_result(lrsa::launch_select(D, score, idx, ws, (hipStream_t)stream), "lrsa_select");
}

int lrsa_check_idx(const lrsa_params* p, const int32_t* idx, int32_t* bad_rows, void* stream) {
    lrsa::Dims D;
    int rc = make_dims(p, &D);
    if (rc != LRSA_OK) return rc;
    if (!bad_rows) return fail(LRSA_ERR_INVALID_ARG, "lrsa_check_idx: bad_rows must not be NULL");
    if (D.Ns > 0 && !idx) return fail(LRSA_ERR_INVALID_ARG, "lrsa_check_idx: idx must not be NULL");
    return hip_result(lrsa::launch_check_idx(D, idx, bad_rows, (hipStream_t)stream), "lrsa_check_idx");
}

int lrsa_score_select(const lrsa_params* p, const void* K, const void* V, float* score, int32_t* idx, void* ws,
                      size_t ws_bytes, void* stream) {
    lrsa::Dims D;
    int rc = make_dims(p, &D);
    if (rc != LRSA_OK) return rc;
    if (D.Ns == 0) return LRSA_OK;
    if (!K || !V || !score || !idx)
        return fail(LRSA_ERR_INVALID_ARG, "lrsa_score_select: K, V, score and idx must not be NULL");
    if (misaligned16(K) || misaligned16(V))
        return fail(LRSA_ERR_INVALID_ARG, "lrsa_score_select: K and V must be 16-byte aligned");
    if ((rc = check_ws(p, D, LRSA_WS_SCORE, ws, ws_bytes)) != LRSA_OK) return rc;
    return hip_result(lrsa::launch_score_select(D, K, V, score, idx, ws, (hipStream_t)stream), "lrsa_score_select");
}

int lrsa_cache_compress(const lrsa_params* p, void* Kc, void* Vc, int32_t* pos, int32_t len, int32_t done,
                        int32_t* len_out, int32_t* done_out, void* stream) {
    lrsa::Dims D;
    int rc = make_dims(p, &D);
    if (rc != LRSA_OK) return rc;
    if (!len_out || !done_out) return fail(LRSA_ERR_INVALID_ARG, "lrsa_cache_compress: len_out and done_out must not be NULL");
    if (!lrsa::cache_compress_supported(D))
        return fail(LRSA_ERR_UNSUPPORTED, "lrsa_cache_compress needs local_prev == 1 and lag <= 4096");
    if (len < 0 || len > D.n || done < 0) return fail(LRSA_ERR_INVALID_ARG, "lrsa_cache_compress: len %d outside [0, cap=%d] or done < 0", len, D.n);
    const int64_t tail = (int64_t)len - D.S - (int64_t)D.K * done;
    if (done > 0 && tail < D.L) return fail(LRSA_ERR_INVALID_ARG, "lrsa_cache_compress: len %d is too short for %d compressed chunks", len, done);
    int steps = tail >= 2 * (int64_t)D.L ? (int)(tail / D.L) - 1 : 0;
    *len_out = len - steps * (D.L - D.K);
    *done_out = done + steps;
    if (steps == 0) return LRSA_OK;
    if (!Kc || !Vc) return fail(LRSA_ERR_INVALID_ARG, "lrsa_cache_compress: Kc and Vc must not be NULL");
    if (misaligned16(Kc) || misaligned16(Vc)) return fail(LRSA_ERR_INVALID_ARG, "lrsa_cache_compress: Kc and Vc must be 16-byte aligned");
    return hip_result(lrsa::launch_cache_compress(D, Kc, Vc, pos, len, done, steps, (hipStream_t)stream), "lrsa_cache_compress");
}

int lrsa_decode_attn(const lrsa_params* p, const void* q, const void* Kc, const void* Vc, int32_t len, void* O,
                     float* lse, void* ws, size_t ws_bytes, void* stream) {
    lrsa::Dims D;
    int rc = make_dims(p, &D);
    if (rc != LRSA_OK) return rc;
    if (len < 1 || len > D.n) return fail(LRSA_ERR_INVALID_ARG, "lrsa_decode_attn: len %d outside [1, cap=%d]", len, D.n);
    if (!q || !Kc || !Vc || !O) return fail(LRSA_ERR_INVALID_ARG, "lrsa_decode_attn: q, Kc, Vc and O must not be NULL");
    if (misaligned16(q) || misaligned16(Kc) || misaligned16(Vc))
        return fail(LRSA_ERR_INVALID_ARG, "lrsa_decode_attn: q, Kc and Vc must be 16-byte aligned");
    if ((rc = check_ws(p, D, LRSA_WS_DECODE_ATTN, ws, ws_bytes)) != LRSA_OK) return rc;
    return hip_result(lrsa::launch_decode_attn(D, q, Kc, Vc, len, O, lse, ws, (hipStream_t)stream), "lrsa_decode_attn");
}

int lrsa_decode_attn_static(const lrsa_params* p, const void* q, const void* Kc, const void* Vc, int32_t len, void* O,
                            float* lse, void* stream) {
    lrsa::Dims D;
    int rc = make_dims(p, &D);
    if (rc != LRSA_OK) return rc;
    if (len < 1 || len > D.n) return fail(LRSA_ERR_INVALID_ARG, "lrsa_decode_attn_static: len %d outside [1, cap=%d]", len, D.n);
    if (!q || !Kc || !Vc || !O) return fail(LRSA_ERR_INVALID_ARG, "lrsa_decode_attn_static: q, Kc, Vc and O must not be NULL");
    if (misaligned16(q) || misaligned16(Kc) || misaligned16(Vc))
        return fail(LRSA_ERR_INVALID_ARG, "lrsa_decode_attn_static: q, Kc and Vc must be 16-byte aligned");
    const size_t need = lrsa::decode_static_need(D, len);
    if (need > lrsa::DECODE_STATIC_SCRATCH_BYTES)
        return fail(LRSA_ERR_INVALID_ARG,
                    "lrsa_decode_attn_static: this call needs %zu bytes of scratch, the built-in array holds %zu "
                    "(batch * heads_q * slices too large); use lrsa_decode_attn with a workspace",
                    need, (size_t)lrsa::DECODE_STATIC_SCRATCH_BYTES);
    return hip_result(lrsa::launch_decode_attn_static(D, q, Kc, Vc, len, O, lse, (hipStream_t)stream), "lrsa_decode_attn_static");
}

int lrsa_attn_fwd(const lrsa_params* p, const void* Q, const void* K, const void* V, const int32_t* idx, void* O,
                  float* lse, void* ws, size_t ws_bytes, void* stream) {
    lrsa::Dims D;
    int rc = make_dims(p, &D);
    if (rc != LRSA_OK) return rc;
    if (!Q || !K || !V || !O || !lse) return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_fwd: Q, K, V, O and lse must not be NULL");
    if (D.Ns > 0 && !idx) return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_fwd: idx is NULL but %d chunks are compressed", D.Ns);
    if (misaligned16(Q) || misaligned16(K) || misaligned16(V) || misaligned16(O))
        return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_fwd: tensors must be 16-byte aligned");
    if ((rc = check_ws(p, D, LRSA_WS_ATTN_FWD, ws, ws_bytes)) != LRSA_OK) return rc;
    const hipError_t e = use_mfma(p, D) ? lrsa::launch_attn_fwd_mfma(D, Q, K, V, idx, O, lse, ws, (hipStream_t)stream)
                                        : lrsa::launch_attn_fwd_generic(D, Q, K, V, idx, O, lse, ws, (hipStream_t)stream);
    return hip_result(e, "lrsa_attn_fwd");
}

int lrsa_attn_bwd(const lrsa_params* p, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                  const float* lse, const int32_t* idx, void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes,
                  void* stream) {
    lrsa::Dims D;
    int rc = make_dims(p, &D);
    if (rc != LRSA_OK) return rc;
    if (!Q || !K || !V || !O || !dO || !lse || !dQ || !dK || !dV)
        return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_bwd: tensor pointers must not be NULL");
    if (D.Ns > 0 && !idx) return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_bwd: idx is NULL but %d chunks are compressed", D.Ns);
    if (misaligned16(Q) || misaligned16(K) || misaligned16(V) || misaligned16(O) || misaligned16(dO) ||
        misaligned16(dQ) || misaligned16(dK) || misaligned16(dV))
        return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_bwd: tensors must be 16-byte aligned");
    if ((rc = check_ws(p, D, LRSA_WS_ATTN_BWD, ws, ws_bytes)) != LRSA_OK) return rc;
    const hipError_t e =
        use_mfma(p, D) ? lrsa::launch_attn_bwd_mfma(D, Q, K, V, O, dO, lse, idx, dQ, dK, dV, nullptr, nullptr, ws, (hipStream_t)stream)
                       : lrsa::launch_attn_bwd_generic(D, Q, K, V, O, dO, lse, idx, dQ, dK, dV, ws, (hipStream_t)stream);
    return hip_result(e, "lrsa_attn_bwd");
}

}  // extern "C"

namespace {

// Row window of one filling step: [row_begin, row_end) must start at 0 or at a chunk start and end at a chunk
// start or at the end of the sequence.  Fills the window fields of the derived dimensions.
int set_row_window(lrsa::Dims* D, int32_t row_begin, int32_t row_end, const char* who) {
    const int n = D->n, S = D->S, L = D->L;
    if (row_begin < 0 || row_end > n || row_begin >= row_end)
        return fail(LRSA_ERR_INVALID_ARG, "%s: rows [%d, %d) are not a window of [0, %d)", who, row_begin, row_end, n);
    const bool begin_ok = row_begin == 0 || (row_begin >= S && (row_begin - S) % L == 0);
    const bool end_ok = row_end == n || (row_end >= S && (row_end - S) % L == 0);
    if (!begin_ok || !end_ok)
        return fail(LRSA_ERR_INVALID_ARG, "%s: rows [%d, %d) do not start and end on chunk boundaries (sink %d, lag %d)", who,
                    row_begin, row_end, S, L);
    D->row_begin = row_begin;
    D->row_end = row_end;
    D->fq0 = row_begin <= S ? 0 : (row_begin - S) / L;
    D->fq1 = row_end == n ? D->nq : (row_end - S) / L;
    D->lse_stride = row_end - row_begin;
    D->compact = 0;     // the condensed copy would be rebuilt at every step: the window calls gather by index
    return LRSA_OK;
}

// base pointer such that row t of the caller's window tensor is addressed as row t of the sequence
const void* shift_rows(const void* p, const lrsa::Dims& D, int64_t row_stride_elems) {
    const int64_t esz = D.dtype == LRSA_BF16 ? 2 : 4;
    return reinterpret_cast<const char*>(p) - int64_t(D.row_begin) * row_stride_elems * esz;
}

}  // namespace

extern "C" {

size_t lrsa_fill_workspace_bytes(const lrsa_params* p, int32_t row_begin, int32_t row_end, int which) {
    lrsa::Dims D;
    if (make_dims(p, &D) != LRSA_OK || !use_mfma(p, D)) return 0;
    if (set_row_window(&D, row_begin, row_end, "lrsa_fill_workspace_bytes") != LRSA_OK) return 0;
    if (which == LRSA_WS_ATTN_FWD) return lrsa::attn_fwd_mfma_ws_bytes(D);
    if (which == LRSA_WS_ATTN_BWD) return lrsa::attn_bwd_mfma_ws_bytes(D);
    return 0;
}

int lrsa_attn_fwd_fill(const lrsa_params* p, int32_t row_begin, int32_t row_end, const void* Q, const void* K,
                       const void* V, const int32_t* idx, void* O, float* lse, void* ws, size_t ws_bytes, void* stream) {
    lrsa::Dims D;
    int rc = make_dims(p, &D);
    if (rc != LRSA_OK) return rc;
    if (!use_mfma(p, D)) return fail(LRSA_ERR_UNSUPPORTED, "lrsa_attn_fwd_fill is built for bf16 with head_dim 128");
    if ((rc = set_row_window(&D, row_begin, row_end, "lrsa_attn_fwd_fill")) != LRSA_OK) return rc;
    if (!Q || !K || !V || !O || !lse) return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_fwd_fill: Q, K, V, O and lse must not be NULL");
    if (D.fq1 - 1 - D.lp > 0 && !idx) return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_fwd_fill: idx is NULL but the rows see compressed chunks");
    if (misaligned16(Q) || misaligned16(K) || misaligned16(V) || misaligned16(O))
        return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_fwd_fill: tensors must be 16-byte aligned");
    const size_t need = lrsa::attn_fwd_mfma_ws_bytes(D);
    if (need > 0 && (!ws || ws_bytes < need)) return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_fwd_fill: workspace of %zu bytes needed", need);
    return hip_result(lrsa::launch_attn_fwd_mfma(D, shift_rows(Q, D, D.qs[2]), K, V, idx,
                                                 const_cast<void*>(shift_rows(O, D, D.qs[2])), lse - D.row_begin, ws,
                                                 (hipStream_t)stream),
                      "lrsa_attn_fwd_fill");
}

int lrsa_attn_bwd_fill(const lrsa_params* p, int32_t row_begin, int32_t row_end, const void* Q, const void* K,
                       const void* V, const void* O, const void* dO, const float* lse, const int32_t* idx, void* dQ,
                       float* dK_acc, float* dV_acc, void* ws, size_t ws_bytes, void* stream) {
    lrsa::Dims D;
    int rc = make_dims(p, &D);
    if (rc != LRSA_OK) return rc;
    if (!use_mfma(p, D)) return fail(LRSA_ERR_UNSUPPORTED, "lrsa_attn_bwd_fill is built for bf16 with head_dim 128");
    if ((rc = set_row_window(&D, row_begin, row_end, "lrsa_attn_bwd_fill")) != LRSA_OK) return rc;
    if (!Q || !K || !V || !O || !dO || !lse || !dQ || !dK_acc || !dV_acc)
        return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_bwd_fill: tensor pointers must not be NULL");
    if (D.fq1 - 1 - D.lp > 0 && !idx) return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_bwd_fill: idx is NULL but the rows see compressed chunks");
    if (misaligned16(Q) || misaligned16(K) || misaligned16(V) || misaligned16(O) || misaligned16(dO) || misaligned16(dQ) ||
        misaligned16(dK_acc) || misaligned16(dV_acc))
        return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_bwd_fill: tensors must be 16-byte aligned");
    const size_t need = lrsa::attn_bwd_mfma_ws_bytes(D);
    if (!ws || ws_bytes < need) return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_bwd_fill: workspace of %zu bytes needed", need);
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return fail(LRSA_ERR_INVALID_ARG, "workspace is not 256-byte aligned");
    D.acc = 1;
    return hip_result(lrsa::launch_attn_bwd_mfma(D, shift_rows(Q, D, D.qs[2]), K, V, shift_rows(O, D, D.qs[2]),
                                                 shift_rows(dO, D, D.qs[2]), lse - D.row_begin, idx,
                                                 const_cast<void*>(shift_rows(dQ, D, D.qs[2])), nullptr, nullptr, dK_acc,
                                                 dV_acc, ws, (hipStream_t)stream),
                      "lrsa_attn_bwd_fill");
}

int lrsa_attn_bwd_finish(const lrsa_params* p, const float* dK_acc, const float* dV_acc, void* dK, void* dV, void* stream) {
    lrsa::Dims D;
    int rc = make_dims(p, &D);
    if (rc != LRSA_OK) return rc;
    if (!use_mfma(p, D)) return fail(LRSA_ERR_UNSUPPORTED, "lrsa_attn_bwd_finish is built for bf16 with head_dim 128");
    if (!dK_acc || !dV_acc || !dK || !dV) return fail(LRSA_ERR_INVALID_ARG, "lrsa_attn_bwd_finish: pointers must not be NULL");
    return hip_result(lrsa::launch_bwd_acc_finish(D, dK_acc, dV_acc, dK, dV, (hipStream_t)stream), "lrsa_attn_bwd_finish");
}

}  // extern "C"
