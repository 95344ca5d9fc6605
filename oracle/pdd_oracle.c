/*
 * pdd_oracle.c -- plain fp64 CPU definition of causal prefill attention and of
 * the observation-window token importance.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file;
 * it exists so that tests, the smoke check and the benchmark's CPU-baseline
 * leg have an independent statement of what the GPU path must compute.  It
 * shares no code, header, table or helper with the HIP library.
 *
 * What is computed (paper, Section 2.2.3, the scaled dot-product attention
 * equation  Attention(Q,K,V) = softmax(Q K^T / sqrt(h)) V ; Section 3.2
 * "Prompt Refiner": the normalised attention weight of the last segment of
 * queries -- the observation window -- against the entire K, summed along the
 * query dimension):
 *
 *   S[i,j]  = scale * sum_c q[i,h,c] * k[j,g,c]      for 0 <= j <= i + delta
 *   m_i     = max_j S[i,j]
 *   Z_i     = sum_j exp(S[i,j] - m_i)
 *   LSE_i   = m_i + ln Z_i
 *   P[i,j]  = exp(S[i,j] - LSE_i)
 *   O[i,h,:] = sum_j P[i,j] * v[j,g,:]
 *   imp[g,j] = sum_{h in group g} sum_{i in window, i + delta >= j} P_h[i,j]
 *
 * with g = h / (Hq/Hkv) (grouped-query attention), delta = Nk - Nq >= 0 (the
 * causal mask is aligned to the bottom-right corner, so a chunk of new queries
 * sees the whole existing prefix), and the window being the last
 * min(W, Nq) queries of each sequence (every query when W < 0).
 *
 * There is no tiling, no running rescale and no re-association: each row is a
 * two-pass softmax over a scratch vector, every dot product is a plain loop.
 * Inputs are bf16 bit patterns, widened exactly to double.
 *
 * Readings where the paper is silent: h is the per-head dimension; the mask is
 * causal (autoregressive prefill); "per head" selection is per KV head with
 * the scores of the group's query heads added.
 *
 * Layouts: q [total_q, Hq, d], k and v [total_k, Hkv, d] (uint16 bf16),
 * cu_q / cu_k int32 [B+1] prefix sums of the per-sequence lengths.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double widen_bf16(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double *widen_array(const uint16_t *src, size_t n)
{
    double *dst = (double *)malloc(sizeof(double) * (n ? n : 1));
    if (!dst) return NULL;
    for (size_t t = 0; t < n; ++t) dst[t] = widen_bf16(src[t]);
    return dst;
}

static int find_sequence(const int32_t *cu, int B, int row)
{
    for (int b = 0; b < B; ++b)
        if (row >= cu[b] && row < cu[b + 1]) return b;
    return -1;
}

static int max_len(const int32_t *cu, int B)
{
    int m = 0;
    for (int b = 0; b < B; ++b)
        if (cu[b + 1] - cu[b] > m) m = cu[b + 1] - cu[b];
    return m;
}

int pddo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* scaled scores of one query row against keys 0..n_vis-1 of its sequence */
static void score_row(const double *qrow, const double *kseq, size_t k_tok_stride,
                      int n_vis, int d, double scale, double *S)
{
    for (int j = 0; j < n_vis; ++j) {
        const double *krow = kseq + (size_t)j * k_tok_stride;
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += qrow[c] * krow[c];
        S[j] = scale * acc;
    }
}

static double log_sum_exp(const double *S, int n)
{
    double m = S[0];
    for (int j = 1; j < n; ++j)
        if (S[j] > m) m = S[j];
    double Z = 0.0;
    for (int j = 0; j < n; ++j) Z += exp(S[j] - m);
    return m + log(Z);
}

/*
 * Attention output and log-sum-exp for selected packed query rows.
 *   rows : n_rows packed query-token indices (NULL = rows 0..n_rows-1)
 *   O    : [n_rows, Hq, d] double ;  lse : [Hq, n_rows] double
 * returns 0, or -1 on a bad argument / allocation failure.
 */
int pddo_attention(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                   int B, int Hq, int Hkv, int d,
                   const int32_t *cu_q, const int32_t *cu_k, double scale,
                   int n_rows, const int32_t *rows, double *O, double *lse)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv) return -1;
    const int G = Hq / Hkv;
    const size_t total_q = (size_t)cu_q[B], total_k = (size_t)cu_k[B];
    double *qd = widen_array(q, total_q * Hq * d);
    double *kd = widen_array(k, total_k * Hkv * d);
    double *vd = widen_array(v, total_k * Hkv * d);
    if (!qd || !kd || !vd) { free(qd); free(kd); free(vd); return -1; }
    const int max_nk = max_len(cu_k, B);
    int status = 0;

#pragma omp parallel
    {
        double *S = (double *)malloc(sizeof(double) * (size_t)(max_nk > 0 ? max_nk : 1));
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int r = 0; r < n_rows; ++r) {
            for (int h = 0; h < Hq; ++h) {
                const int row = rows ? rows[r] : r;
                const int b = find_sequence(cu_q, B, row);
                if (b < 0 || !S) {
#pragma omp atomic write
                    status = -1;
                    continue;
                }
                const int nq = cu_q[b + 1] - cu_q[b], nk = cu_k[b + 1] - cu_k[b];
                const int delta = nk - nq;
                const int i = row - cu_q[b];
                const int n_vis = i + delta + 1;          /* keys 0 .. i+delta */
                const int g = h / G;
                const size_t kstride = (size_t)Hkv * d;
                const double *qrow = qd + ((size_t)row * Hq + h) * d;
                const double *kseq = kd + ((size_t)cu_k[b] * Hkv + g) * d;
                const double *vseq = vd + ((size_t)cu_k[b] * Hkv + g) * d;
                double *out = O + ((size_t)r * Hq + h) * d;
                if (delta < 0 || n_vis <= 0) {
#pragma omp atomic write
                    status = -1;
                    continue;
                }
                score_row(qrow, kseq, kstride, n_vis, d, scale, S);
                const double L = log_sum_exp(S, n_vis);
                lse[(size_t)h * n_rows + r] = L;
                for (int c = 0; c < d; ++c) out[c] = 0.0;
                for (int j = 0; j < n_vis; ++j) {
                    const double p = exp(S[j] - L);
                    const double *vrow = vseq + (size_t)j * kstride;
                    for (int c = 0; c < d; ++c) out[c] += p * vrow[c];
                }
            }
        }
        free(S);
    }
    free(qd); free(kd); free(vd);
    return status;
}

/*
 * Token importance: imp [Hkv, total_k] double, every entry written.
 * window < 0 : every query of a sequence is a window query (chunk mode).
 * window >= 0: the last min(window, Nq) queries.
 * Phase 1 gets LSE_i of every (head, window row) from the definition; phase 2
 * evaluates P[i,j] = exp(S[i,j] - LSE_i) per key and adds in a fixed order
 * (heads of the group ascending, window rows ascending).
 */
int pddo_importance(const uint16_t *q, const uint16_t *k,
                    int B, int Hq, int Hkv, int d,
                    const int32_t *cu_q, const int32_t *cu_k, double scale,
                    int window, double *imp)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv) return -1;
    const int G = Hq / Hkv;
    const size_t total_q = (size_t)cu_q[B], total_k = (size_t)cu_k[B];
    double *qd = widen_array(q, total_q * Hq * d);
    double *kd = widen_array(k, total_k * Hkv * d);
    if (!qd || !kd) { free(qd); free(kd); return -1; }
    const int max_nk = max_len(cu_k, B), max_nq = max_len(cu_q, B);
    const size_t kstride = (size_t)Hkv * d;
    int status = 0;
    for (size_t t = 0; t < (size_t)Hkv * total_k; ++t) imp[t] = 0.0;

    for (int b = 0; b < B && status == 0; ++b) {
        const int nq = cu_q[b + 1] - cu_q[b], nk = cu_k[b + 1] - cu_k[b];
        const int delta = nk - nq;
        if (delta < 0) { status = -1; break; }
        if (nq == 0) continue;
        const int W = (window < 0 || window > nq) ? nq : window;
        if (W == 0) continue;
        const int i0 = nq - W;
        double *L = (double *)malloc(sizeof(double) * (size_t)Hq * W);
        if (!L) { status = -1; break; }
        (void)max_nq;

        /* phase 1: log-sum-exp of every window row */
#pragma omp parallel
        {
            double *S = (double *)malloc(sizeof(double) * (size_t)(max_nk > 0 ? max_nk : 1));
#pragma omp for collapse(2) schedule(dynamic, 1)
            for (int h = 0; h < Hq; ++h) {
                for (int w = 0; w < W; ++w) {
                    const int i = i0 + w;
                    const int n_vis = i + delta + 1;
                    const double *qrow = qd + ((size_t)(cu_q[b] + i) * Hq + h) * d;
                    const double *kseq = kd + ((size_t)cu_k[b] * Hkv + h / G) * d;
                    score_row(qrow, kseq, kstride, n_vis, d, scale, S);
                    L[(size_t)h * W + w] = log_sum_exp(S, n_vis);
                }
            }
            free(S);
        }

        /* phase 2: column sums of the normalised window weights */
#pragma omp parallel for collapse(2) schedule(dynamic, 64)
        for (int g = 0; g < Hkv; ++g) {
            for (int j = 0; j < nk; ++j) {
                const double *krow = kd + ((size_t)(cu_k[b] + j) * Hkv + g) * d;
                double acc = 0.0;
                for (int h = g * G; h < (g + 1) * G; ++h) {
                    for (int w = 0; w < W; ++w) {
                        const int i = i0 + w;
                        if (j > i + delta) continue;          /* causally masked */
                        const double *qrow = qd + ((size_t)(cu_q[b] + i) * Hq + h) * d;
                        double s = 0.0;
                        for (int c = 0; c < d; ++c) s += qrow[c] * krow[c];
                        acc += exp(scale * s - L[(size_t)h * W + w]);
                    }
                }
                imp[(size_t)g * total_k + cu_k[b] + j] = acc;
            }
        }
        free(L);
    }
    free(qd); free(kd);
    return status;
}
