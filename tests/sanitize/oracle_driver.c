/* Driver for the sanitizer pass over the C part of the CPU checker: runs pddo_attention and
 * pddo_importance on small seeded problems that exercise the ragged, empty-sequence, chunked,
 * grouped-head and window-longer-than-prompt paths and prints a checksum of every output.  The
 * test builds it twice, plain and with AddressSanitizer + UndefinedBehaviorSanitizer, and
 * requires identical output and a clean exit. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int pddo_attention(const uint16_t *q, const uint16_t *k, const uint16_t *v, int B, int Hq, int Hkv, int d,
                   const int32_t *cu_q, const int32_t *cu_k, double scale, int n_rows, const int32_t *rows,
                   double *O, double *lse);
int pddo_importance(const uint16_t *q, const uint16_t *k, int B, int Hq, int Hkv, int d, const int32_t *cu_q,
                    const int32_t *cu_k, double scale, int window, double *imp);

static uint32_t lcg_state = 12345u;
static uint16_t next_bf16(void)
{
    /* a small finite bf16 value: sign, exponent 120..127, 7 mantissa bits */
    lcg_state = lcg_state * 1664525u + 1013904223u;
    const uint32_t r = lcg_state >> 8;
    return (uint16_t)(((r & 1u) << 15) | ((120u + ((r >> 1) & 7u)) << 7) | ((r >> 4) & 127u));
}

static double checksum(const double *x, size_t n)
{
    double s = 0.0;
    for (size_t i = 0; i < n; ++i) s += x[i] * (double)(1 + (i % 7));
    return s;
}

static int run_case(const char *name, int B, const int32_t *len_q, const int32_t *len_k, int Hq, int Hkv, int d,
                    int window, int n_rows, const int32_t *rows)
{
    int32_t cu_q[16], cu_k[16];
    cu_q[0] = cu_k[0] = 0;
    for (int b = 0; b < B; ++b) { cu_q[b + 1] = cu_q[b] + len_q[b]; cu_k[b + 1] = cu_k[b] + len_k[b]; }
    const size_t tq = (size_t)cu_q[B], tk = (size_t)cu_k[B];
    uint16_t *q = malloc(sizeof(uint16_t) * (tq * Hq * d + 1)), *k = malloc(sizeof(uint16_t) * (tk * Hkv * d + 1)),
             *v = malloc(sizeof(uint16_t) * (tk * Hkv * d + 1));
    for (size_t i = 0; i < tq * Hq * d; ++i) q[i] = next_bf16();
    for (size_t i = 0; i < tk * Hkv * d; ++i) k[i] = next_bf16();
    for (size_t i = 0; i < tk * Hkv * d; ++i) v[i] = next_bf16();
    const size_t nr = rows ? (size_t)n_rows : tq;
    double *O = malloc(sizeof(double) * (nr * Hq * d + 1)), *lse = malloc(sizeof(double) * (nr * Hq + 1)),
           *imp = malloc(sizeof(double) * (tk * Hkv + 1));
    int rc = pddo_attention(q, k, v, B, Hq, Hkv, d, cu_q, cu_k, 0.125, (int)nr, rows, O, lse);
    rc |= pddo_importance(q, k, B, Hq, Hkv, d, cu_q, cu_k, 0.125, window, imp);
    printf("%s rc=%d O=%.17g lse=%.17g imp=%.17g\n", name, rc, checksum(O, nr * Hq * d), checksum(lse, nr * Hq),
           checksum(imp, tk * Hkv));
    free(q); free(k); free(v); free(O); free(lse); free(imp);
    return rc;
}

int main(void)
{
    int bad = 0;
    { const int32_t l[4] = {37, 0, 1, 70};  bad |= run_case("ragged", 4, l, l, 4, 2, 16, 50, 0, NULL); }
    { const int32_t lq[3] = {5, 33, 1}, lk[3] = {5 + 40, 33, 1 + 64};  bad |= run_case("chunked", 3, lq, lk, 6, 2, 8, -1, 0, NULL); }
    { const int32_t l[1] = {129};  const int32_t rows[5] = {0, 1, 64, 127, 128};  bad |= run_case("rows", 1, l, l, 2, 2, 64, 8, 5, rows); }
    { const int32_t l[2] = {3, 2};  bad |= run_case("mha-tiny", 2, l, l, 3, 3, 4, 1, 0, NULL); }
    /* argument errors are reported, not followed */
    { const int32_t cu[2] = {0, 4};  double x[8];  uint16_t z[64] = {0};
      if (pddo_attention(z, z, z, 1, 3, 2, 4, cu, cu, 1.0, 4, NULL, x, x) == 0) { printf("bad head grouping accepted\n"); bad = 1; } }
    return bad ? 1 : 0;
}
