/* CPU oracle for LRSA attention at sizes where a dense n x n matrix does not fit --
 * TEST INFRASTRUCTURE ONLY, never linked or loaded by the product library.
 *
 * The same definition as the NumPy oracle (attention = softmax(Q K^T / sqrt(d_h) + M) V,
 * Eq. 2-3 of the paper, under the chunked mask of the "Attention Filling" steps), written
 * as loops over one query row or one key column at a time so that single rows / columns
 * of a long sequence can be evaluated.  fp64 arithmetic on fp32-held inputs.  No tiling,
 * no online softmax: every row materialises its logits, subtracts the maximum,
 * exponentiates and normalises.
 *
 * One call works on one (batch, KV head): Q and dO hold the G query heads of that group
 * as [G][n][d], K and V are [n][d], idx is [Ns][K] (absolute positions, may be NULL when
 * Ns == 0).  OpenMP only spreads independent rows / columns over threads.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t G, n, d, S, L, K, Ns, local_prev;
    double scale;
} lrsa_oracle_cfg;

/* selected[u] = 1 when position u survived the compression of its chunk */
static unsigned char *build_selected(const lrsa_oracle_cfg *c, const int32_t *idx)
{
    unsigned char *sel = (unsigned char *)calloc((size_t)c->n, 1);
    if (sel && idx)
        for (int64_t i = 0; i < (int64_t)c->Ns * c->K; ++i) sel[idx[i]] = 1;
    return sel;
}

/* the mask: causal, and sink / sink query / local window / survivor */
static int visible(const lrsa_oracle_cfg *c, const unsigned char *sel, int64_t t, int64_t u)
{
    if (u > t) return 0;
    if (u < c->S || t < c->S) return 1;
    int64_t ct = (t - c->S) / c->L, cu = (u - c->S) / c->L;
    if (cu >= ct - c->local_prev) return 1;
    return sel[u];
}

static double dot(const float *a, const float *b, int d)
{
    double acc = 0.0;
#pragma omp simd reduction(+ : acc)
    for (int c = 0; c < d; ++c) acc += (double)a[c] * (double)b[c];
    return acc;
}

/* Forward (and dQ) for the listed query rows.
 * Outputs, indexed [g][r] over the G heads and the nrows listed rows:
 *   O [G][nrows][d], lse [G][nrows]; when dO != NULL also D = rowsum(dO*O) [G][nrows]
 *   and, unless dQ is NULL (a caller that wants lse and D only), dQ [G][nrows][d] =
 *   scale * sum_u dS[t,u] k_u with dS = A (dA - D).
 * Returns 0, or -1 when memory runs out. */
int lrsa_oracle_rows(const lrsa_oracle_cfg *c, const float *Q, const float *K, const float *V,
                     const float *dO, const int32_t *idx, const int64_t *rows, int64_t nrows,
                     double *O, double *lse, double *D, double *dQ)
{
    unsigned char *sel = build_selected(c, idx);
    if (!sel) return -1;
    const int d = c->d;
    int failed = 0;
#pragma omp parallel
    {
        double *logit = (double *)malloc(sizeof(double) * (size_t)c->n);
        int64_t *key = (int64_t *)malloc(sizeof(int64_t) * (size_t)c->n);
        if (!logit || !key) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for collapse(2) schedule(dynamic, 4)
            for (int g = 0; g < c->G; ++g)
                for (int64_t r = 0; r < nrows; ++r) {
                    const int64_t t = rows[r];
                    const float *q = Q + ((int64_t)g * c->n + t) * d;
                    int64_t m = 0;
                    double mx = -INFINITY;
                    for (int64_t u = 0; u <= t; ++u)
                        if (visible(c, sel, t, u)) {
                            key[m] = u;
                            logit[m] = c->scale * dot(q, K + u * d, d);
                            if (logit[m] > mx) mx = logit[m];
                            ++m;
                        }
                    double den = 0.0;
                    for (int64_t j = 0; j < m; ++j) {
                        logit[j] = exp(logit[j] - mx);
                        den += logit[j];
                    }
                    double *o = O + ((int64_t)g * nrows + r) * d;
                    for (int x = 0; x < d; ++x) o[x] = 0.0;
                    for (int64_t j = 0; j < m; ++j) {
                        logit[j] /= den; /* attention weight A[t, key[j]] */
                        const float *v = V + key[j] * d;
                        for (int x = 0; x < d; ++x) o[x] += logit[j] * (double)v[x];
                    }
                    lse[(int64_t)g * nrows + r] = mx + log(den);
                    if (dO) {
                        const float *go = dO + ((int64_t)g * c->n + t) * d;
                        double Dt = 0.0;
                        for (int x = 0; x < d; ++x) Dt += (double)go[x] * o[x];
                        D[(int64_t)g * nrows + r] = Dt;
                        if (!dQ) continue;
                        double *dq = dQ + ((int64_t)g * nrows + r) * d;
                        for (int x = 0; x < d; ++x) dq[x] = 0.0;
                        for (int64_t j = 0; j < m; ++j) {
                            const double dA = dot(go, V + key[j] * d, d);
                            const double dS = logit[j] * (dA - Dt);
                            const float *k = K + key[j] * d;
                            for (int x = 0; x < d; ++x) dq[x] += c->scale * dS * (double)k[x];
                        }
                    }
                }
        }
        free(logit);
        free(key);
    }
    free(sel);
    return failed ? -1 : 0;
}

/* dK and dV for the listed key columns, [ncols][d] each, summed over the G heads.
 * lse_all and D_all are [G][n]; only entries of rows that see a listed column are read.
 *   dV[u] = sum_t A[t,u] dO_t,  dK[u] = scale * sum_t dS[t,u] q_t,
 *   A[t,u] = exp(scale q_t.k_u - lse_t), dS = A (dO_t.v_u - D_t). */
int lrsa_oracle_cols(const lrsa_oracle_cfg *c, const float *Q, const float *K, const float *V,
                     const float *dO, const int32_t *idx, const double *lse_all, const double *D_all,
                     const int64_t *cols, int64_t ncols, double *dK, double *dV)
{
    unsigned char *sel = build_selected(c, idx);
    if (!sel) return -1;
    const int d = c->d;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t j = 0; j < ncols; ++j) {
        const int64_t u = cols[j];
        const float *k = K + u * d, *v = V + u * d;
        double *dk = dK + j * d, *dv = dV + j * d;
        for (int x = 0; x < d; ++x) dk[x] = dv[x] = 0.0;
        for (int g = 0; g < c->G; ++g)
            for (int64_t t = u; t < c->n; ++t) {
                if (!visible(c, sel, t, u)) continue;
                const float *q = Q + ((int64_t)g * c->n + t) * d;
                const float *go = dO + ((int64_t)g * c->n + t) * d;
                const double A = exp(c->scale * dot(q, k, d) - lse_all[(int64_t)g * c->n + t]);
                const double dS = A * (dot(go, v, d) - D_all[(int64_t)g * c->n + t]);
                for (int x = 0; x < d; ++x) {
                    dv[x] += A * (double)go[x];
                    dk[x] += c->scale * dS * (double)q[x];
                }
            }
    }
    free(sel);
    return 0;
}

/* Number of keys row t sees, by counting the mask (pins the closed-form count). */
int64_t lrsa_oracle_count(const lrsa_oracle_cfg *c, const int32_t *idx, int64_t t)
{
    unsigned char *sel = build_selected(c, idx);
    if (!sel) return -1;
    int64_t m = 0;
    for (int64_t u = 0; u <= t; ++u) m += visible(c, sel, t, u);
    free(sel);
    return m;
}
