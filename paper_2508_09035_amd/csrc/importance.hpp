// Token importance from the observation window (paper Section 3.2, "Prompt
// Refiner": the normalised attention weight of the last segment of queries
// against the entire K, summed along the query dimension).
//
//   imp[g, j] = sum_{h in group g} sum_{i in window, i + delta >= j}
//               exp(s <q_i, k_j> - lse[h, i])
//
// The final log-sum-exp of every window row is an input, so each probability
// is recomputed from one QK^T tile and added into a per-key column sum; the
// attention matrix is never stored.  Work is split over KEYS: a wave owns 32
// keys, keeps their K fragments in registers (B operand) and sweeps all window
// rows of all G query heads (A operand, streamed from L2).  S = Q K^T puts key
// (l % 32) in lane l and 16 query rows in its accumulator registers, so the
// sum over queries is in-lane; no atomics, fixed summation order.
#pragma once
#include "attn_fwd.hpp"

namespace pdd {

struct ImpParams {
    const uint16_t *q, *k;
    const float *lse;
    float *imp;
    const int32_t *cu_q, *cu_k;
    int64_t q_st, q_sh, k_st, k_sh;
    int32_t B, Hq, Hkv, G, total_q, total_k, n_ktiles;
    int32_t window;    // < 0: every query is a window query
    float scale_log2;  // softmax scale * log2(e)
};

constexpr int kImpWaves = 4;
constexpr int kImpBK = 32 * kImpWaves;  // keys per workgroup

template <int D>
__global__ __launch_bounds__(kImpWaves * 64) void importance_kernel(const ImpParams p)
{
    constexpr int NKK = D / 16;
    int bid = blockIdx.x;
    const int g = bid % p.Hkv;  bid /= p.Hkv;
    const int b = bid % p.B;    bid /= p.B;
    const int kt = bid;

    const int qs = min(p.cu_q[b], p.total_q), qe = min(p.cu_q[b + 1], p.total_q);
    const int ks = min(p.cu_k[b], p.total_k), ke = min(p.cu_k[b + 1], p.total_k);
    const int nq = qe - qs, nk = ke - ks;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, hh = lane >> 5;
    const int jw0 = kt * kImpBK + 32 * wave;   // first key of this wave
    if (jw0 >= nk) return;
    const int j = jw0 + n;
    const int delta = nk - nq;
    const int W = (p.window < 0 || p.window > nq) ? nq : p.window;
    const int iw0 = nq - W;                    // first window row

    // K fragments (B operand): key j, dims 16*kk + 8*hh .. +7
    bf16x8 kf[NKK];
    {
        const uint16_t *kp = p.k + (int64_t)(ks + min(j, nk - 1)) * p.k_st + (int64_t)g * p.k_sh + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) kf[kk] = *(const bf16x8 *)(kp + 16 * kk);
    }
    const float c2 = p.scale_log2;
    constexpr float kLog2e = 1.4426950408889634f;
    float colsum = 0.f;

    if (nq > 0 && delta >= 0) {
        // first row block that can see key jw0: rows i >= jw0 - delta
        const int rb_first = max(0, (jw0 - delta - iw0) / 32);
        const int n_rb = (W + 31) / 32;
        for (int hg = 0; hg < p.G; ++hg) {
            const int h = g * p.G + hg;
            const float *lse_h = p.lse + (int64_t)h * p.total_q + qs;
            for (int rb = rb_first; rb < n_rb; ++rb) {
                const int i0 = iw0 + 32 * rb;
                const int irow = min(i0 + n, nq - 1);   // A operand row of this lane
                const uint16_t *qp = p.q + (int64_t)(qs + irow) * p.q_st + (int64_t)h * p.q_sh + 8 * hh;
                f32x16 s;
#pragma unroll
                for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
                for (int kk = 0; kk < NKK; ++kk) {
                    const bf16x8 a = *(const bf16x8 *)(qp + 16 * kk);
                    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, kf[kk], s, 0, 0, 0);
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int i = i0 + 8 * (e >> 2) + 4 * hh + (e & 3);
                    const bool ok = (i < nq) && (j <= i + delta) && (j < nk);
                    const float l2 = lse_h[min(i, nq - 1)] * kLog2e;
                    const float pr = fast_exp2(fmaf(s[e], c2, -l2));
                    colsum += ok ? pr : 0.f;
                }
            }
        }
    }
    colsum += xchg_half(colsum);
    if (hh == 0 && j < nk) p.imp[(int64_t)g * p.total_k + ks + j] = colsum;
}

}  // namespace pdd
