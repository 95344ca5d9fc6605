// Sentence-level selection (paper Section 3.2, "Prompt Refiner": the KV cache
// entries of one sentence are combined and treated as a whole, so that
// selecting KV cache entries means selecting sentences; Section 1: sentence-
// level selection keeps the refined prompt semantically coherent).
//
// Per (sequence, head row): sentences are contiguous token ranges that tile the
// content part [cand_begin, sent_end[last]).  A sentence's score is the sum or
// the mean of its tokens' scores; sentences are ranked by (score descending,
// index ascending) and the longest prefix of that ranking whose token count
// fits the budget is kept.  Outputs: keep flag per sentence, 0/1 mask per
// token, number of kept tokens.
//
// One 1024-thread workgroup per row.  Sentence sums are serial fp32 loops in
// token order (deterministic); ranks come from counting in LDS (S^2 / 1024
// compares per thread, S <= 8192 sentences); the kept prefix from a block
// scan of the lengths in rank order; the token mask from a binary search of
// the sentence ends.
#pragma once
#include "select_topk.hpp"

namespace pdd {

enum { kSentSum = 0, kSentMean = 1 };
constexpr int kSentMax = 8192;    // sentences per sequence held in LDS

struct SentParams {
    const float *scores;
    const int32_t *cu_k, *cu_sent, *sent_end, *cand_b, *budget;
    uint8_t *sent_keep, *mask;
    int32_t *kept_tokens;
    float *sent_scores;
    int32_t n_heads, B, total_k, total_sent, s_cap, mode;
};

__global__ __launch_bounds__(kSelThreads) void select_sentences_kernel(const SentParams p)
{
    extern __shared__ __attribute__((aligned(16))) int32_t sent_smem[];
    int32_t *send = sent_smem;                       // [s_cap] clamped sentence ends
    uint32_t *skey = (uint32_t *)(send + p.s_cap);   // [s_cap] order keys, later keep flags
    int32_t *slen = (int32_t *)(skey + p.s_cap);     // [s_cap] token counts
    int32_t *lenr = slen + p.s_cap;                  // [s_cap] lengths in rank order -> inclusive scan
    __shared__ int32_t wsum[kSelWaves];
    __shared__ int32_t sh_m;

    const int b = blockIdx.x, g = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ks = min(max(p.cu_k[b], 0), p.total_k);
    const int ke = min(max(p.cu_k[b + 1], ks), p.total_k);
    const int nk = ke - ks;
    const int s0 = min(max(p.cu_sent[b], 0), p.total_sent);
    const int s1 = min(max(p.cu_sent[b + 1], s0), p.total_sent);
    const int S = min(s1 - s0, p.s_cap);
    const int c0 = min(max(p.cand_b ? p.cand_b[b] : 0, 0), nk);
    const int budget = max(p.budget[b], 0);
    const float *seq = p.scores + (int64_t)g * p.total_k + ks;
    uint8_t *mrow = p.mask ? p.mask + (int64_t)g * p.total_k + ks : nullptr;

    // sentence ends, forced into [c0, nk] and non-decreasing (serial fix-up by one thread is
    // avoided: an end smaller than its predecessor is raised by a running maximum below)
    for (int s = tid; s < S; s += kSelThreads) send[s] = min(max(p.sent_end[s0 + s], c0), nk);
    __syncthreads();
    // running maximum over at most a few thousand entries: wave 0, 64 lanes, chunked
    if (wave == 0) {
        const int ch = (S + 63) / 64;
        const int lo = lane * ch, hi = min(lo + ch, S);
        int mx = c0;
        for (int s = lo; s < hi; ++s) mx = max(mx, send[s]);
        int run = mx;                                  // inclusive max over lanes <= lane
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(run, off, 64);
            if (lane >= off) run = max(run, o);
        }
        int prev = __shfl_up(run, 1, 64);
        if (lane == 0) prev = c0;
        for (int s = lo; s < hi; ++s) { prev = max(prev, send[s]); send[s] = prev; }
    }
    __syncthreads();
    const int content_end = S > 0 ? send[S - 1] : c0;

    // sentence scores
    for (int s = tid; s < S; s += kSelThreads) {
        const int st = s == 0 ? c0 : send[s - 1], en = send[s];
        float acc = 0.f;
        for (int x = st; x < en; ++x) acc += seq[x];
        const int len = en - st;
        const float sc = (p.mode == kSentMean) ? acc / (float)max(len, 1) : acc;
        skey[s] = order_key(sc);
        slen[s] = len;
        if (p.sent_scores) p.sent_scores[(int64_t)g * p.total_sent + s0 + s] = sc;
    }
    __syncthreads();

    // ranks by counting; lengths scattered into rank order
    constexpr int OWN = kSentMax / kSelThreads;        // sentences per thread at most
    int my_rank[OWN];
#pragma unroll
    for (int i = 0; i < OWN; ++i) {
        const int s = i * kSelThreads + tid;
        my_rank[i] = 0;
        if (s < S) {
            const uint32_t ksv = skey[s];
            int beats = 0;
            for (int t = 0; t < S; ++t) {
                const uint32_t kt = skey[t];
                beats += (kt > ksv || (kt == ksv && t < s)) ? 1 : 0;
            }
            my_rank[i] = beats;
            lenr[beats] = slen[s];
        }
    }
    __syncthreads();

    // inclusive scan of lenr[0..S): contiguous chunk per thread
    const int ch = (S + kSelThreads - 1) / kSelThreads;
    const int lo = min(tid * ch, S), hi = min(lo + ch, S);
    int local = 0;
    for (int r = lo; r < hi; ++r) local += lenr[r];
    int incl = local;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(incl, off, 64);
        if (lane >= off) incl += o;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    int base = incl - local;
    for (int w = 0; w < wave; ++w) base += wsum[w];
    int cnt_fit = 0;
    for (int r = lo; r < hi; ++r) {
        base += lenr[r];
        lenr[r] = base;                                  // cumulative token count of ranks 0..r
        cnt_fit += base <= budget ? 1 : 0;
    }
    // m = number of leading ranks that fit (the cumulative counts are non-decreasing)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) cnt_fit += __shfl_xor(cnt_fit, off, 64);
    __syncthreads();
    if (lane == 0) wsum[wave] = cnt_fit;
    __syncthreads();
    if (tid == 0) {
        int m = 0;
        for (int w = 0; w < kSelWaves; ++w) m += wsum[w];
        sh_m = m;
        if (p.kept_tokens) p.kept_tokens[(int64_t)g * p.B + b] = m > 0 ? lenr[m - 1] : 0;
    }
    __syncthreads();
    const int m = sh_m;

    // keep flags
#pragma unroll
    for (int i = 0; i < OWN; ++i) {
        const int s = i * kSelThreads + tid;
        if (s < S) {
            const uint32_t kept = my_rank[i] < m ? 1u : 0u;
            skey[s] = kept;
            if (p.sent_keep) p.sent_keep[(int64_t)g * p.total_sent + s0 + s] = (uint8_t)kept;
        }
    }
    __syncthreads();

    // token mask: token x of the content belongs to the first sentence whose end is > x
    if (mrow) {
        for (int x = tid; x < nk; x += kSelThreads) {
            uint8_t v = 0;
            if (x >= c0 && x < content_end) {
                int a = 0, z = S - 1;                    // send[z] > x holds for z = S - 1
                while (a < z) {
                    const int mid = (a + z) >> 1;
                    if (send[mid] > x) z = mid; else a = mid + 1;
                }
                v = (uint8_t)skey[a];
            }
            mrow[x] = v;
        }
    }
}

}  // namespace pdd
