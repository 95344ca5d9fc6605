// Top-k token selection and stable index compaction (paper Section 3.2,
// "Prompt Refiner": the indices with the top summed scores are kept at ratio
// r and the positions are filtered; the mask tensor has 1 at position i when
// token i is selected).
//
// One workgroup per (sequence, head) row.  The k-th largest score is found by
// a 4 x 8-bit most-significant-first radix select on order-preserving integer
// images of the fp32 scores (LDS histograms); ties at the threshold are
// resolved towards the lower index.  The kept indices are then written in
// ascending order by a ballot / popcount compaction (each wave owns a
// contiguous slice, so the output order is the index order).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pdd {

struct SelParams {
    const float *scores;
    const int32_t *cu_k, *cand_b, *cand_e, *k_per, *cu_keep;
    int32_t *out_idx;
    uint8_t *out_mask;
    int32_t n_heads, B, total_k, total_keep;
    int32_t lds_cap;   // scores staged per row (STAGED variant): longer rows are truncated
};

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelLdsCap = 32768;   // scores staged in LDS up to this row length

__device__ __forceinline__ uint32_t order_key(float x)
{
    // monotone map fp32 -> uint32 (larger float <=> larger key); -0.0 == +0.0
    const uint32_t u = __float_as_uint(x + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <bool STAGED>
__device__ __forceinline__ uint32_t sel_key(const uint32_t *skeys, const float *row, int idx)
{
    return STAGED ? skeys[idx] : order_key(row[idx]);
}

template <bool STAGED>
__global__ __launch_bounds__(kSelThreads) void select_topk_kernel(const SelParams p)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t sel_smem[];
    __shared__ uint32_t hist[256];
    __shared__ int32_t sh_bin, sh_above;
    __shared__ int32_t wave_gt[kSelWaves], wave_eq[kSelWaves];
    uint32_t *skeys = sel_smem;

    const int b = blockIdx.x, g = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ks = min(max(p.cu_k[b], 0), p.total_k);
    const int ke = min(max(p.cu_k[b + 1], ks), p.total_k);
    const int nk = ke - ks;
    int c0 = p.cand_b ? p.cand_b[b] : 0;
    int c1 = p.cand_e ? p.cand_e[b] : nk;
    c0 = min(max(c0, 0), nk);
    c1 = min(max(c1, c0), nk);
    const int n = STAGED ? min(c1 - c0, p.lds_cap) : c1 - c0;
    const int keep0 = min(max(p.cu_keep[b], 0), p.total_keep);
    const int keep1 = min(max(p.cu_keep[b + 1], keep0), p.total_keep);
    const int slots = keep1 - keep0;
    const int kk = min(min(max(p.k_per[b], 0), n), slots);

    const float *row = p.scores + (int64_t)g * p.total_k + ks + c0;
    int32_t *out = p.out_idx + (int64_t)g * p.total_keep + keep0;
    uint8_t *mrow = p.out_mask ? p.out_mask + (int64_t)g * p.total_k + ks : nullptr;

    // mask outside the candidate range, unused index slots
    if (mrow) {
        for (int x = tid; x < c0; x += kSelThreads) mrow[x] = 0;
        for (int x = c1 + tid; x < nk; x += kSelThreads) mrow[x] = 0;
    }
    for (int x = kk + tid; x < slots; x += kSelThreads) out[x] = -1;
    if (kk == 0) {
        if (mrow)
            for (int x = c0 + tid; x < c1; x += kSelThreads) mrow[x] = 0;
        return;
    }

    if (STAGED) {
        for (int x = tid; x < n; x += kSelThreads) skeys[x] = order_key(row[x]);
    }

    // ---- radix select: after the loop `prefix` is the key of the kk-th largest
    uint32_t prefix = 0, pmask = 0;
    int krem = kk;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int x0 = 0; x0 < n; x0 += kSelThreads) {
            const int x = x0 + tid;
            const bool in = x < n;
            const uint32_t key = in ? sel_key<STAGED>(skeys, row, x) : 0u;
            const bool part = in && ((key & pmask) == prefix);
            const uint32_t bin = (key >> shift) & 255u;
            // one round of wave aggregation: lanes that share the first
            // participating lane's bin are counted with a single atomic
            const uint64_t pm = __ballot(part);
            if (pm) {
                const int leader = __ffsll((unsigned long long)pm) - 1;
                const uint32_t lbin = __shfl(bin, leader, 64);
                const uint64_t same = __ballot(part && bin == lbin);
                if (lane == leader) atomicAdd(&hist[lbin], (uint32_t)__popcll(same));
                if (part && bin != lbin) atomicAdd(&hist[bin], 1u);
            }
        }
        __syncthreads();
        if (wave == 0) {
            // lane L owns bins 4L .. 4L+3 ; `above` = count in bins greater than d
            uint32_t c[4];
            uint32_t s = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) { c[i] = hist[4 * lane + i]; s += c[i]; }
            uint32_t incl = s;   // inclusive suffix sum over lanes >= L
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t o = __shfl_down(incl, off, 64);
                if (lane + off < 64) incl += o;
            }
            uint32_t above = incl - s;
#pragma unroll
            for (int i = 3; i >= 0; --i) {
                if ((uint32_t)krem > above && (uint32_t)krem <= above + c[i]) {
                    sh_bin = 4 * lane + i;
                    sh_above = (int32_t)above;
                }
                above += c[i];
            }
        }
        __syncthreads();
        prefix |= ((uint32_t)sh_bin) << shift;
        pmask |= 255u << shift;
        krem -= sh_above;
        __syncthreads();
    }
    const uint32_t T = prefix;   // threshold key; `krem` (>= 1) ties at T are kept, lowest index first

    // ---- stable compaction: each wave owns a contiguous slice of the candidates
    const int seg = ((n + kSelWaves - 1) / kSelWaves + 63) & ~63;
    const int s0 = min(wave * seg, n), s1 = min(s0 + seg, n);
    int cgt = 0, ceq = 0;
    for (int x0 = s0; x0 < s1; x0 += 64) {
        const int x = x0 + lane;
        const bool in = x < s1;
        const uint32_t key = in ? sel_key<STAGED>(skeys, row, x) : 0u;
        cgt += __popcll(__ballot(in && key > T));
        ceq += __popcll(__ballot(in && key == T));
    }
    if (lane == 0) { wave_gt[wave] = cgt; wave_eq[wave] = ceq; }
    __syncthreads();
    int gt_before = 0, eq_before = 0;
    for (int w = 0; w < wave; ++w) { gt_before += wave_gt[w]; eq_before += wave_eq[w]; }
    int sel_before = gt_before + min(eq_before, krem);
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    for (int x0 = s0; x0 < s1; x0 += 64) {
        const int x = x0 + lane;
        const bool in = x < s1;
        const uint32_t key = in ? sel_key<STAGED>(skeys, row, x) : 0u;
        const bool is_gt = in && key > T, is_eq = in && key == T;
        const uint64_t be = __ballot(is_eq);
        const int eq_rank = eq_before + __popcll(be & lt_mask);
        const bool sel = is_gt || (is_eq && eq_rank < krem);
        const uint64_t bs = __ballot(sel);
        if (sel) out[sel_before + __popcll(bs & lt_mask)] = c0 + x;
        if (mrow && in) mrow[c0 + x] = sel ? 1 : 0;
        sel_before += __popcll(bs);
        eq_before += __popcll(be);
    }
}

}  // namespace pdd
