// Top-k token selection and stable index compaction (paper Section 3.2,
// "Prompt Refiner": the indices with the top summed scores are kept at ratio
// r and the positions are filtered; the mask tensor has 1 at position i when
// token i is selected).
//
// One workgroup of 1024 threads per (sequence, head) row; scores become
// order-preserving uint32 keys.  Two kernels:
//
//  * select_topk_reg_kernel<EPT> (rows of up to 1024*EPT <= 32768 candidates):
//    every thread keeps its EPT keys in registers for the whole kernel.  The
//    k-th largest key is found by bisection on the key value inside the row's
//    [min, max] range: one step = EPT compares per lane, wave ballots counted
//    on the scalar unit, one 16-entry LDS exchange.  No LDS atomics (measured
//    at ~30 cycles per wave instruction, they dominated the radix variant)
//    and no re-reading of the row.  The kept indices are written in ascending
//    order from ballot prefix counts, with a 16*EPT-entry scan across waves.
//  * select_topk_kernel (longer rows): most-significant-first radix select,
//    8 bits per pass, digits taken from (key - min key) scaled to the row's
//    range, LDS histograms; the row is re-read from L2 in every pass.
//
// Ties at the threshold are resolved towards the lower index in both.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pdd {

enum { kPoolNone = 0, kPoolMax = 1, kPoolAvg = 2 };

struct SelParams {
    const float *scores;
    const int32_t *cu_k, *cand_b, *cand_e, *k_per, *cu_keep;
    int32_t *out_idx;
    uint8_t *out_mask;
    int32_t n_heads, B, total_k, total_keep;
    int32_t pool_r, pool_mode;   // 1-D pooling radius (kernel = 2r+1) and kPool* mode; r = 0: none
    float pool_inv;              // 1 / kernel for the average
    float *pooled_out;           // optional [n_heads, total_k]: the pooled scores that were ranked
};

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelFinish = 64;    // keys left in the bracket that are ranked directly
constexpr int kSelRegCap = 32 * 1024;  // rows up to this many candidates stay in registers

// Score of key j after 1-D pooling along the sequence (paper Section 3.2: a pooling step
// between the sum over queries and the sort, so that neighbours are kept together).  Window = keys
// [j-r, j+r] inside the sequence; max over the valid part, or sum of the valid part divided by
// the kernel size (zero padding).  seq = first score of the sequence row, nk = its length.
__device__ __forceinline__ float pooled_score(const float *seq, int nk, int j, int r, int mode, float inv)
{
    if (r == 0) return seq[j];
    const int lo = max(j - r, 0), hi = min(j + r, nk - 1);
    float acc = seq[lo];
    if (mode == kPoolMax) {
        for (int t = lo + 1; t <= hi; ++t) acc = fmaxf(acc, seq[t]);
        return acc;
    }
    for (int t = lo + 1; t <= hi; ++t) acc += seq[t];
    return acc * inv;
}

__device__ __forceinline__ uint32_t order_key(float x)
{
    // monotone map fp32 -> uint32 (larger float <=> larger key); -0.0 == +0.0
    const uint32_t u = __float_as_uint(x + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}


// ---------------------------------------------------------------------------
// Register-resident selection for rows of at most 1024 * EPT candidates.
// Thread `tid` owns candidates x = i * 1024 + tid, i = 0 .. EPT-1.
// ---------------------------------------------------------------------------
// POOL = false: the instantiation for unpooled scores carries none of the pooling code.
template <int EPT, bool POOL>
__global__ __launch_bounds__(kSelThreads) void select_topk_reg_kernel(const SelParams p)
{
    __shared__ uint32_t wred[2][kSelWaves];            // per-wave partial counts (double buffered)
    __shared__ uint32_t wave_min[kSelWaves], wave_max[kSelWaves];
    __shared__ uint32_t cnt[kSelWaves * EPT];          // per (i, wave): gt count | eq count << 16
    __shared__ uint32_t cnt_wave_tot[kSelWaves];
    __shared__ uint32_t fin_keys[kSelFinish], fin_count, fin_T, fin_above;

    const int b = blockIdx.x, g = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ks = min(max(p.cu_k[b], 0), p.total_k);
    const int ke = min(max(p.cu_k[b + 1], ks), p.total_k);
    const int nk = ke - ks;
    int c0 = p.cand_b ? p.cand_b[b] : 0;
    int c1 = p.cand_e ? p.cand_e[b] : nk;
    c0 = min(max(c0, 0), nk);
    c1 = min(max(c1, c0), nk);
    const int n = min(c1 - c0, kSelThreads * EPT);
    const int keep0 = min(max(p.cu_keep[b], 0), p.total_keep);
    const int keep1 = min(max(p.cu_keep[b + 1], keep0), p.total_keep);
    const int slots = keep1 - keep0;
    const int kk = min(min(max(p.k_per[b], 0), n), slots);

    const float *seq = p.scores + (int64_t)g * p.total_k + ks;
    int32_t *out = p.out_idx + (int64_t)g * p.total_keep + keep0;
    uint8_t *mrow = p.out_mask ? p.out_mask + (int64_t)g * p.total_k + ks : nullptr;

    if (p.pooled_out) {
        float *po = p.pooled_out + (int64_t)g * p.total_k + ks;
        if constexpr (POOL) {
            for (int x = tid; x < nk; x += kSelThreads) po[x] = pooled_score(seq, nk, x, p.pool_r, p.pool_mode, p.pool_inv);
        } else {
            for (int x = tid; x < nk; x += kSelThreads) po[x] = seq[x];
        }
    }
    if (mrow) {
        for (int x = tid; x < c0; x += kSelThreads) mrow[x] = 0;
        for (int x = c0 + n + tid; x < nk; x += kSelThreads) mrow[x] = 0;
    }
    for (int x = kk + tid; x < slots; x += kSelThreads) out[x] = -1;
    if (kk == 0) {
        if (mrow)
            for (int x = c0 + tid; x < c0 + n; x += kSelThreads) mrow[x] = 0;
        return;
    }

    // ---- keys into registers; row range
    uint32_t key[EPT];
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    if constexpr (!POOL) {
        // plain loads from clamped (always valid: n >= 1 here) addresses, so that all of them are
        // in flight before the first one is used
        float raw[EPT];
#pragma unroll
        for (int i = 0; i < EPT; ++i) raw[i] = seq[c0 + min(i * kSelThreads + tid, n - 1)];
#pragma unroll
        for (int i = 0; i < EPT; ++i) key[i] = (i * kSelThreads + tid < n) ? order_key(raw[i]) : 0u;
    } else {
#pragma unroll
        for (int i = 0; i < EPT; ++i) {
            const int x = i * kSelThreads + tid;
            key[i] = x < n ? order_key(pooled_score(seq, nk, c0 + x, p.pool_r, p.pool_mode, p.pool_inv)) : 0u;
        }
    }
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        const bool in = i * kSelThreads + tid < n;
        kmin = in ? min(kmin, key[i]) : kmin;
        kmax = in ? max(kmax, key[i]) : kmax;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, off, 64));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off, 64));
    }
    if (lane == 0) { wave_min[wave] = kmin; wave_max[wave] = kmax; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) { kmin = min(kmin, wave_min[w]); kmax = max(kmax, wave_max[w]); }

    // ---- threshold search: largest T in [kmin, kmax] with count(key >= T) >= kk.
    // Bisection on the key value with the bracket [lo, hi] and the two counts
    // c_lo = count(key >= lo) >= kk > c_above = count(key > hi); once at most kSelFinish keys
    // are left inside the bracket they are collected in LDS and ranked directly (about 12
    // probes instead of 27 for a row of 32768; probing the point where a straight line through
    // the two counts crosses kk was tried and needs more probes: it converges from one side).
    // Invalid slots hold key 0 and every probed T is > kmin >= 0, so they never count.
    uint32_t lo = kmin, hi = kmax;
    uint32_t c_lo = (uint32_t)n;       // count(key >= lo)
    uint32_t c_above = 0;              // count(key >= hi + 1) = count(key > T) at the end
    int par = 0;
    while (lo < hi && c_lo - c_above > (uint32_t)kSelFinish) {
        const uint32_t mid = lo + ((hi - lo + 1u) >> 1);
        uint32_t c = 0;
#pragma unroll
        for (int i = 0; i < EPT; ++i) c += (uint32_t)__popcll(__ballot(key[i] >= mid));
        if (lane == 0) wred[par][wave] = c;
        __syncthreads();
        uint32_t tot = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) tot += wred[par][w];
        par ^= 1;
        if (tot >= (uint32_t)kk) { lo = mid; c_lo = tot; }
        else { hi = mid - 1u; c_above = tot; }
    }
    if (lo < hi) {
        // at most kSelFinish keys lie in [lo, hi]: the (kk - c_above)-th largest of them is T
        if (tid == 0) fin_count = 0;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < EPT; ++i) {
            const bool in = i * kSelThreads + tid < n;
            if (in && key[i] >= lo && key[i] <= hi) {
                const uint32_t slot = atomicAdd(&fin_count, 1u);
                if (slot < (uint32_t)kSelFinish) fin_keys[slot] = key[i];
            }
        }
        __syncthreads();
        if (wave == 0) {
            const uint32_t m = min(fin_count, (uint32_t)kSelFinish);
            const uint32_t mine_k = lane < (int)m ? fin_keys[lane] : 0u;
            uint32_t gt = 0, ge = 0;
            for (uint32_t j = 0; j < m; ++j) {
                const uint32_t o = fin_keys[j];
                gt += o > mine_k ? 1u : 0u;
                ge += o >= mine_k ? 1u : 0u;
            }
            const uint32_t r = (uint32_t)kk - c_above;                    // 1 <= r <= m
            const bool hit = lane < (int)m && gt < r && r <= ge;          // every hit lane holds the same key
            const uint64_t hb = __ballot(hit);
            if (hb != 0 && lane == (int)__builtin_ctzll(hb)) { fin_T = mine_k; fin_above = c_above + gt; }
        }
        __syncthreads();
        lo = fin_T;
        c_above = fin_above;
    }
    const uint32_t T = lo;
    const int krem = kk - (int)c_above;     // ties at T to keep (>= 1), lowest index first

    // ---- per (i, wave) counts of keys > T and == T, scanned in index order (i major, wave minor)
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        const bool in = i * kSelThreads + tid < n;
        const uint32_t cg = (uint32_t)__popcll(__ballot(in && key[i] > T));
        const uint32_t ce = (uint32_t)__popcll(__ballot(in && key[i] == T));
        if (lane == i) mine = cg | (ce << 16);
    }
    if (lane < EPT) cnt[lane * kSelWaves + wave] = mine;
    __syncthreads();
    constexpr int NC = kSelWaves * EPT;                 // <= 512 entries, one per thread
    uint32_t v = tid < NC ? cnt[tid] : 0u, incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = (uint32_t)__shfl_up((int)incl, off, 64);
        if (lane >= off) incl += o;
    }
    if (lane == 63) cnt_wave_tot[wave] = incl;
    __syncthreads();
    uint32_t wave_off = 0;
    for (int w = 0; w < wave; ++w) wave_off += cnt_wave_tot[w];
    if (tid < NC) cnt[tid] = wave_off + incl - v;       // exclusive prefix (packed gt | eq << 16)
    __syncthreads();

    // ---- stable compaction
    const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        const int x = i * kSelThreads + tid;
        const bool in = x < n;
        const uint32_t before = cnt[i * kSelWaves + wave];
        const int gt_before = (int)(before & 0xffffu), eq_before = (int)(before >> 16);
        const bool is_gt = in && key[i] > T, is_eq = in && key[i] == T;
        const uint64_t be = __ballot(is_eq);
        const int eq_rank = eq_before + __popcll(be & lt_mask);
        const bool sel = is_gt || (is_eq && eq_rank < krem);
        const uint64_t bs = __ballot(sel);
        const int sel_before = gt_before + min(eq_before, krem);
        if (sel) out[sel_before + __popcll(bs & lt_mask)] = c0 + x;
        if (mrow && in) mrow[c0 + x] = sel ? 1 : 0;
    }
}

// ---------------------------------------------------------------------------
// Register-resident selection, four consecutive candidates per lane and step (unpooled scores
// from a 16-byte aligned tensor).  Thread `tid` owns the quads q = i * 1024 + tid, i < QPT, of
// the row's 16-byte aligned part (the up to three candidates before the first 16-byte boundary
// sit one each in the first lanes of wave 0).  Against the one-candidate-per-lane kernel above: 16-byte loads, the mask written four bytes at a time, and a threshold
// search that leaves the block-wide probes (each one costs a barrier) as soon as the keys still
// in the bracket fit into one wave's registers; that wave finishes the bisection on its own.
// ---------------------------------------------------------------------------
constexpr int kSelWaveKeys = 2048;     // bracket size at which one wave takes over (32 keys per lane)

// inclusive prefix sum over the 64 lanes of a wave (DPP row shifts and row broadcasts)
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x)
{
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, true);   // row_shr:1
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, true);   // row_shr:2
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, true);   // row_shr:4
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, true);   // row_shr:8
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1, 3
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2, 3
    return x;
}

// Next value to probe in the threshold search over the bracket [lo, hi] (lo < hi) that holds
// `inside` keys, of which the `need` largest (1 <= need <= inside) lie at or above the threshold.
// With interpolate set, the keys are taken as evenly spread over the bracket, which is nearly true
// once the bracket is a narrow slice of the score distribution, and the probe lands a few keys
// away from the threshold instead of halving the bracket; otherwise the bracket is bisected.  The
// callers interpolate as long as the previous probe cut the number of keys in the bracket to a
// quarter or less and bisect after one that did not, which bounds the worst case at twice the
// probes of plain bisection.  The result is in [lo + 1, hi]: either outcome shrinks the bracket.
__device__ __forceinline__ uint32_t next_probe(uint32_t lo, uint32_t hi, uint32_t inside, uint32_t need, bool interpolate)
{
    const uint32_t span = hi - lo;
    if (!interpolate) return lo + ((span + 1u) >> 1);
    const float f = ((float)need - 0.5f) / (float)inside;          // share of the bracket above the threshold
    const uint32_t down = (uint32_t)min(f * (float)span, 4294967040.f);
    return hi - min(down, span - 1u);
}

template <int QPT>
__global__ __launch_bounds__(kSelThreads) void select_topk_quad_kernel(const SelParams p)
{
    __shared__ uint32_t wred[2][kSelWaves];
    __shared__ uint32_t wave_min[kSelWaves], wave_max[kSelWaves];
    __shared__ uint32_t cnt[kSelWaves * QPT];          // per (i, wave): gt count | eq count << 16
    __shared__ uint32_t cnt_wave_tot[kSelWaves];
    __shared__ uint32_t fin_keys[kSelWaveKeys];
    __shared__ uint32_t fin_T, fin_above, head_tot;

    const int b = blockIdx.x, g = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ks = min(max(p.cu_k[b], 0), p.total_k);
    const int ke = min(max(p.cu_k[b + 1], ks), p.total_k);
    const int nk = ke - ks;
    int c0 = p.cand_b ? p.cand_b[b] : 0;
    int c1 = p.cand_e ? p.cand_e[b] : nk;
    c0 = min(max(c0, 0), nk);
    c1 = min(max(c1, c0), nk);
    const int n = min(c1 - c0, 4 * kSelThreads * QPT);
    // Candidates 0 .. nhead-1 (at most three) precede the first 16-byte boundary of the row; lanes
    // 0 .. nhead-1 of wave 0 hold one each.  Candidate nhead + 4q + j is element j of quad q.
    const int64_t elem0 = (int64_t)g * p.total_k + ks + c0;      // first candidate, in elements of `scores`
    const int nhead = min((int)((4 - (elem0 & 3)) & 3), n);
    const int nq_el = n - nhead;                                 // candidates inside quads
    const int keep0 = min(max(p.cu_keep[b], 0), p.total_keep);
    const int keep1 = min(max(p.cu_keep[b + 1], keep0), p.total_keep);
    const int slots = keep1 - keep0;
    const int kk = min(min(max(p.k_per[b], 0), n), slots);

    const float *seq = p.scores + (int64_t)g * p.total_k + ks;
    int32_t *out = p.out_idx + (int64_t)g * p.total_keep + keep0;
    uint8_t *mrow = p.out_mask ? p.out_mask + (int64_t)g * p.total_k + ks : nullptr;

    if (p.pooled_out) {
        float *po = p.pooled_out + (int64_t)g * p.total_k + ks;
        for (int x = tid; x < nk; x += kSelThreads) po[x] = seq[x];
    }
    if (mrow) {
        for (int x = tid; x < c0; x += kSelThreads) mrow[x] = 0;
        for (int x = c0 + n + tid; x < nk; x += kSelThreads) mrow[x] = 0;
    }
    for (int x = kk + tid; x < slots; x += kSelThreads) out[x] = -1;
    if (kk == 0) {
        if (mrow)
            for (int x = c0 + tid; x < c0 + n; x += kSelThreads) mrow[x] = 0;
        return;
    }

    // ---- keys into registers.  Slots outside the row hold key 0, which is below the key of
    // every finite score.
    const bool has_head = tid < nhead;
    const uint32_t khead = has_head ? order_key(seq[c0 + tid]) : 0u;
    const float *qbase = seq + c0 + nhead;                       // 16-byte aligned
    uint32_t key[QPT][4];
#pragma unroll
    for (int i = 0; i < QPT; ++i) {
        const int x0 = 4 * (i * kSelThreads + tid);              // index inside the quad part
        float f[4] = {0.f, 0.f, 0.f, 0.f};
        if (x0 + 3 < nq_el) {
            const float4 t = *(const float4 *)(qbase + x0);
            f[0] = t.x;  f[1] = t.y;  f[2] = t.z;  f[3] = t.w;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (x0 + j < nq_el) f[j] = qbase[x0 + j];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) key[i][j] = (x0 + j < nq_el) ? order_key(f[j]) : 0u;
    }
    uint32_t kmin = has_head ? khead : 0xffffffffu, kmax = khead;
#pragma unroll
    for (int i = 0; i < QPT; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool in = 4 * (i * kSelThreads + tid) + j < nq_el;
            kmin = in ? min(kmin, key[i][j]) : kmin;
            kmax = max(kmax, key[i][j]);
        }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, off, 64));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off, 64));
    }
    if (lane == 0) { wave_min[wave] = kmin; wave_max[wave] = kmax; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) { kmin = min(kmin, wave_min[w]); kmax = max(kmax, wave_max[w]); }

    // ---- threshold search, block-wide part: bisection on the key value as in the kernel above,
    // until at most kSelWaveKeys keys are left in the bracket [lo, hi]; every probed value is
    // > lo >= kmin > 0, so empty slots never count.
    uint32_t lo = kmin, hi = kmax;
    uint32_t c_lo = (uint32_t)n, c_above = 0;
    int par = 0;
    bool interp = true;
    while (lo < hi && c_lo - c_above > (uint32_t)kSelWaveKeys) {
        const uint32_t inside = c_lo - c_above;
        const uint32_t mid = next_probe(lo, hi, inside, (uint32_t)kk - c_above, interp);
        uint32_t c = (uint32_t)__popcll(__ballot(khead >= mid));
#pragma unroll
        for (int i = 0; i < QPT; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) c += (uint32_t)__popcll(__ballot(key[i][j] >= mid));
        if (lane == 0) wred[par][wave] = c;
        __syncthreads();
        uint32_t tot = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) tot += wred[par][w];
        par ^= 1;
        if (tot >= (uint32_t)kk) { lo = mid; c_lo = tot; }
        else { hi = mid - 1u; c_above = tot; }
        interp = !interp || 4u * (c_lo - c_above) <= inside;
    }
    if (lo < hi) {
        // ---- the keys still inside [lo, hi] (at most kSelWaveKeys) go to LDS, in any order ...
        // (lo >= kmin > 0: empty slots are outside the bracket)
        uint32_t mine = (khead >= lo && khead <= hi) ? 1u : 0u;
#pragma unroll
        for (int i = 0; i < QPT; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) mine += (key[i][j] >= lo && key[i][j] <= hi) ? 1u : 0u;
        const uint32_t incl = wave_incl_scan(mine);
        if (lane == 63) cnt_wave_tot[wave] = incl;
        __syncthreads();
        uint32_t pos = incl - mine, m_tot = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) {               // independent reads, no trip count to wait for
            const uint32_t t = cnt_wave_tot[w];
            pos += w < wave ? t : 0u;
            m_tot += t;
        }
        if (khead >= lo && khead <= hi) fin_keys[pos++] = khead;
#pragma unroll
        for (int i = 0; i < QPT; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (key[i][j] >= lo && key[i][j] <= hi) fin_keys[pos++] = key[i][j];
        __syncthreads();
        // ---- ... and one wave, KPL of them per lane, continues the bisection without barriers
        // until at most kSelFinish keys are left, which it ranks directly: the r-th largest of
        // the m_tot keys, r = kk - c_above
        if (wave == 0) {
            constexpr int KPL = kSelWaveKeys / 64;
            uint32_t fk[KPL];
#pragma unroll
            for (int t = 0; t < KPL; ++t) fk[t] = (t * 64 + lane) < (int)m_tot ? fin_keys[t * 64 + lane] : 0u;
            const uint32_t r = (uint32_t)kk - c_above;              // 1 <= r <= m_tot
            uint32_t wlo = lo, whi = hi;
            uint32_t w_ge = m_tot, above = 0;                       // count(key >= wlo), count(key > whi)
            bool winterp = true;
            while (wlo < whi && w_ge - above > (uint32_t)kSelFinish) {
                const uint32_t inside = w_ge - above;
                const uint32_t mid = next_probe(wlo, whi, inside, r - above, winterp);
                // per-lane counts on four independent chains, one wave sum at the end (a ballot and
                // a scalar population count per key would wait for each other with one wave running)
                uint32_t cl[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int t = 0; t < KPL; ++t) cl[t & 3] += fk[t] >= mid ? 1u : 0u;
                const uint32_t c = (uint32_t)__builtin_amdgcn_readlane(
                    (int)wave_incl_scan((cl[0] + cl[1]) + (cl[2] + cl[3])), 63);
                if (c >= r) { wlo = mid; w_ge = c; }
                else { whi = mid - 1u; above = c; }
                winterp = !winterp || 4u * (w_ge - above) <= inside;
            }
            uint32_t T_w = wlo;
            if (wlo < whi) {
                // the keys inside [wlo, whi] (at most kSelFinish) in the first LDS slots, then the
                // (r - above)-th largest of them by counting
                const uint64_t lt_mask = (1ull << lane) - 1ull;
                uint32_t m = 0;
#pragma unroll
                for (int t = 0; t < KPL; ++t) {
                    const bool inb = fk[t] >= wlo && fk[t] <= whi;      // empty slots hold 0 < wlo
                    const uint64_t bal = __ballot(inb);
                    if (inb) fin_keys[m + __popcll(bal & lt_mask)] = fk[t];
                    m += (uint32_t)__popcll(bal);
                }
                const uint32_t mine_k = lane < (int)m ? fin_keys[lane] : 0u;
                uint32_t gt = 0, ge = 0;
                for (uint32_t j = 0; j < m; ++j) {
                    const uint32_t o = fin_keys[j];
                    gt += o > mine_k ? 1u : 0u;
                    ge += o >= mine_k ? 1u : 0u;
                }
                const uint32_t rr = r - above;                             // 1 <= rr <= m
                const bool hit = lane < (int)m && gt < rr && rr <= ge;     // every hit lane holds the same key
                const uint64_t hb = __ballot(hit);
                const int src = hb ? (int)__builtin_ctzll(hb) : 0;
                T_w = (uint32_t)__shfl((int)mine_k, src, 64);
                above += (uint32_t)__shfl((int)gt, src, 64);
            }
            if (lane == 0) { fin_T = T_w; fin_above = c_above + above; }
        }
        __syncthreads();
        lo = fin_T;
        c_above = fin_above;
    }
    const uint32_t T = lo;
    const int krem = kk - (int)c_above;     // ties at T to keep (>= 1), lowest index first

    // ---- counts of keys > T and == T in index order: the head, then (i major, lane, j)
    const uint32_t c_head = (has_head && khead > T ? 1u : 0u) | (has_head && khead == T ? 0x10000u : 0u);
    uint32_t pre_head = 0;                  // wave 0: exclusive prefix over the head lanes
    if (wave == 0) {
        const uint32_t incl = wave_incl_scan(c_head);
        pre_head = incl - c_head;
        if (lane == 63) head_tot = incl;
    }
    uint32_t pre[QPT];                      // exclusive prefix inside the wave, packed gt | eq << 16
#pragma unroll
    for (int i = 0; i < QPT; ++i) {
        uint32_t c = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {                  // empty slots hold key 0 < kmin <= T
            c += key[i][j] > T ? 1u : 0u;
            c += key[i][j] == T ? 0x10000u : 0u;
        }
        const uint32_t incl = wave_incl_scan(c);
        pre[i] = incl - c;
        if (lane == 63) cnt[i * kSelWaves + wave] = incl;
    }
    __syncthreads();
    constexpr int NC = kSelWaves * QPT;                 // <= 128 entries
    {
        const uint32_t v = tid < NC ? cnt[tid] : 0u;
        const uint32_t incl = wave_incl_scan(v);
        if (lane == 63) cnt_wave_tot[wave] = incl;
        __syncthreads();
        uint32_t wave_off = head_tot;
        for (int w = 0; w < wave; ++w) wave_off += cnt_wave_tot[w];
        if (tid < NC) cnt[tid] = wave_off + incl - v;   // exclusive prefix over the head and (i, wave)
        __syncthreads();
    }

    // ---- stable compaction
    if (has_head) {
        const int gt_before = (int)(pre_head & 0xffffu), eq_before = (int)(pre_head >> 16);
        const bool sel = khead > T || (khead == T && eq_before < krem);
        if (sel) out[gt_before + min(eq_before, krem)] = c0 + tid;
        if (mrow) mrow[c0 + tid] = sel ? 1 : 0;
    }
#pragma unroll
    for (int i = 0; i < QPT; ++i) {
        const int x0 = 4 * (i * kSelThreads + tid);
        const uint32_t before = cnt[i * kSelWaves + wave] + pre[i];
        int gt_before = (int)(before & 0xffffu), eq_before = (int)(before >> 16);
        uint32_t mbytes = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool is_gt = key[i][j] > T, is_eq = key[i][j] == T;    // never true for an empty slot
            const bool sel = is_gt || (is_eq && eq_before < krem);
            if (sel) out[gt_before + min(eq_before, krem)] = c0 + nhead + x0 + j;
            gt_before += is_gt ? 1 : 0;
            eq_before += is_eq ? 1 : 0;
            mbytes |= sel ? (1u << (8 * j)) : 0u;
        }
        if (mrow && x0 < nq_el) {
            uint8_t *mp = mrow + c0 + nhead + x0;                          // 4-byte aligned
            if (x0 + 3 < nq_el) *(uint32_t *)mp = mbytes;
            else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (x0 + j < nq_el) mp[j] = (uint8_t)((mbytes >> (8 * j)) & 1u);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Radix selection for rows longer than 32768 candidates (keys re-read from L2).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kSelThreads) void select_topk_kernel(const SelParams p)
{
    __shared__ uint32_t hist[256];
    __shared__ int32_t sh_bin, sh_above;
    __shared__ int32_t wave_gt[kSelWaves], wave_eq[kSelWaves];

    const int b = blockIdx.x, g = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ks = min(max(p.cu_k[b], 0), p.total_k);
    const int ke = min(max(p.cu_k[b + 1], ks), p.total_k);
    const int nk = ke - ks;
    int c0 = p.cand_b ? p.cand_b[b] : 0;
    int c1 = p.cand_e ? p.cand_e[b] : nk;
    c0 = min(max(c0, 0), nk);
    c1 = min(max(c1, c0), nk);
    const int n = c1 - c0;
    const int keep0 = min(max(p.cu_keep[b], 0), p.total_keep);
    const int keep1 = min(max(p.cu_keep[b + 1], keep0), p.total_keep);
    const int slots = keep1 - keep0;
    const int kk = min(min(max(p.k_per[b], 0), n), slots);

    const float *seq = p.scores + (int64_t)g * p.total_k + ks;
    int32_t *out = p.out_idx + (int64_t)g * p.total_keep + keep0;
    uint8_t *mrow = p.out_mask ? p.out_mask + (int64_t)g * p.total_k + ks : nullptr;
    auto cand_key = [&](int x) {
        return order_key(pooled_score(seq, nk, c0 + x, p.pool_r, p.pool_mode, p.pool_inv));
    };

    if (p.pooled_out) {
        float *po = p.pooled_out + (int64_t)g * p.total_k + ks;
        for (int x = tid; x < nk; x += kSelThreads) po[x] = pooled_score(seq, nk, x, p.pool_r, p.pool_mode, p.pool_inv);
    }
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

    // ---- the row's key range
    __shared__ uint32_t wave_min[kSelWaves], wave_max[kSelWaves];
    uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll 8
    for (int x = tid; x < n; x += kSelThreads) {
        const uint32_t key = cand_key(x);
        kmin = min(kmin, key);
        kmax = max(kmax, key);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, off, 64));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off, 64));
    }
    if (lane == 0) { wave_min[wave] = kmin; wave_max[wave] = kmax; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) { kmin = min(kmin, wave_min[w]); kmax = max(kmax, wave_max[w]); }
    const uint32_t range = kmax - kmin;
    const int nbits = 32 - __builtin_clz(range | 1u);        // 1 .. 32
    const int passes = (nbits + 7) >> 3;                     // 1 .. 4
    const int lsh = 8 * passes - nbits;                      // scaled key = (key - kmin) << lsh < 2^(8 passes)
    const bool aggregate = nbits < 12;

    // ---- radix select on the scaled keys: afterwards `prefix` is the scaled key of the kk-th largest
    uint32_t prefix = 0;
    int krem = kk;
    for (int pass = 0; pass < passes; ++pass) {
        const int shift = 8 * (passes - 1 - pass);
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
#pragma unroll 4
        for (int x0 = 0; x0 < n; x0 += kSelThreads) {
            const int x = x0 + tid;
            const bool in = x < n;
            const uint32_t sk = in ? (cand_key(x) - kmin) << lsh : 0u;
            // digits above the current one must equal the prefix found so far
            const bool part = in && (pass == 0 || (sk >> (shift + 8)) == prefix);
            const uint32_t bin = (sk >> shift) & 255u;
            if (!aggregate) {
                // wide key range: the scaled digits spread over the bins, plain LDS atomics
                if (part) atomicAdd(&hist[bin], 1u);
            } else {
                // narrow range (many equal keys): lanes that share the first participating
                // lane's bin are counted with a single atomic
                const uint64_t pm = __ballot(part);
                if (pm) {
                    const int leader = __ffsll((unsigned long long)pm) - 1;
                    const uint32_t lbin = __builtin_amdgcn_readlane(bin, leader);
                    const uint64_t same = __ballot(part && bin == lbin);
                    if (lane == leader) atomicAdd(&hist[lbin], (uint32_t)__popcll(same));
                    if (part && bin != lbin) atomicAdd(&hist[bin], 1u);
                }
            }
        }
        __syncthreads();
        if (wave == 0) {
            // lane L owns bins 4L .. 4L+3 ; `above` = count in bins greater than d
            uint32_t c[4];
            uint32_t sum4 = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) { c[i] = hist[4 * lane + i]; sum4 += c[i]; }
            uint32_t incl = sum4;   // inclusive suffix sum over lanes >= L
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t o = __shfl_down(incl, off, 64);
                if (lane + off < 64) incl += o;
            }
            uint32_t above = incl - sum4;
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
        prefix = (prefix << 8) | (uint32_t)sh_bin;
        krem -= sh_above;
        __syncthreads();
    }
    const uint32_t T = kmin + (prefix >> lsh);   // threshold key; `krem` (>= 1) ties at T are kept, lowest index first

    // ---- stable compaction: each wave owns a contiguous slice of the candidates
    const int seg = ((n + kSelWaves - 1) / kSelWaves + 63) & ~63;
    const int s0 = min(wave * seg, n), s1 = min(s0 + seg, n);
    int cgt = 0, ceq = 0;
    for (int x0 = s0; x0 < s1; x0 += 64) {
        const int x = x0 + lane;
        const bool in = x < s1;
        const uint32_t key = in ? cand_key(x) : 0u;
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
        const uint32_t key = in ? cand_key(x) : 0u;
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
