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
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);    // negative: all bits flipped; else the sign bit set
}


// ---------------------------------------------------------------------------
// Register-resident selection for rows of at most 4096 * QPT candidates, four consecutive
// candidates per lane and step.  Thread `tid` owns the quads q = i * 1024 + tid, i < QPT, of the
// row's part that starts at a 16-byte boundary of the score tensor (the up to three candidates
// before it sit one each in the first lanes of wave 0): 16-byte loads, the mask written four
// bytes at a time where the mask tensor's alignment allows it.
// POOL = true ranks the 1-D pooled scores (evaluated while loading; no 16-byte loads then);
// the instantiation for unpooled scores carries none of the pooling code.
// ---------------------------------------------------------------------------
constexpr int kSelMaxProbes = 72;       // a 32-bit bracket needs at most 2 x 32 probes (see next_probe)

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

// the same over N independent values per lane, one step over all of them at a time: consecutive
// instructions are independent, so none of them waits for the DPP hazard of its predecessor
template <int N>
__device__ __forceinline__ void wave_incl_scan_n(uint32_t (&x)[N])
{
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x[i], 0x111, 0xf, 0xf, true);
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x[i], 0x112, 0xf, 0xf, true);
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x[i], 0x114, 0xf, 0xf, true);
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x[i], 0x118, 0xf, 0xf, true);
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x[i], 0x142, 0xa, 0xf, false);
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x[i], 0x143, 0xc, 0xf, false);
}

// minimum / maximum over the 64 lanes of a wave, valid in lane 63 (same DPP pattern as the scan)
__device__ __forceinline__ void wave_min_max(uint32_t &mn, uint32_t &mx)
{
    // lanes without a source keep their own value (old = the value itself)
#define PDD_MINMAX_STEP(CTRL, ROWS)                                                                         \
    {                                                                                                       \
        const uint32_t a = (uint32_t)__builtin_amdgcn_update_dpp((int)mn, (int)mn, CTRL, ROWS, 0xf, false); \
        const uint32_t b = (uint32_t)__builtin_amdgcn_update_dpp((int)mx, (int)mx, CTRL, ROWS, 0xf, false); \
        mn = min(mn, a);                                                                                    \
        mx = max(mx, b);                                                                                    \
    }
    PDD_MINMAX_STEP(0x111, 0xf)
    PDD_MINMAX_STEP(0x112, 0xf)
    PDD_MINMAX_STEP(0x114, 0xf)
    PDD_MINMAX_STEP(0x118, 0xf)
    PDD_MINMAX_STEP(0x142, 0xa)
    PDD_MINMAX_STEP(0x143, 0xc)
#undef PDD_MINMAX_STEP
}

// At most 64 vector registers, so that two workgroups (8 waves per SIMD) share a compute unit: the
// kernel lives on overlapping one row's barriers and latencies with another row's work
// (512 rows of 32768: 2.29 TB/s with two workgroups per compute unit, 1.85 with one).
template <int QPT, bool POOL>
__global__ __launch_bounds__(kSelThreads) __attribute__((amdgpu_waves_per_eu(8, 8)))
void select_topk_reg_kernel(const SelParams p)
{
    __shared__ uint32_t wave_min[kSelWaves], wave_max[kSelWaves];
    __shared__ uint32_t cnt[kSelWaves * QPT];          // per (i, wave): gt count | eq count << 16
    __shared__ uint32_t probe_tot[kSelMaxProbes];      // count of probe number p, summed over the waves
    __shared__ __attribute__((aligned(16))) uint32_t fin_keys[kSelFinish + 4];
    __shared__ uint32_t fin_count, fin_T, fin_above, head_tot;

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
    const float *seq = p.scores + (int64_t)g * p.total_k + ks;
    const int nhead = POOL ? 0 : min((int)(((16u - ((uint32_t)(uintptr_t)(seq + c0) & 15u)) & 15u) >> 2), n);
    const int nq_el = n - nhead;                                 // candidates inside quads
    const int keep0 = min(max(p.cu_keep[b], 0), p.total_keep);
    const int keep1 = min(max(p.cu_keep[b + 1], keep0), p.total_keep);
    const int slots = keep1 - keep0;
    const int kk = min(min(max(p.k_per[b], 0), n), slots);

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

    // ---- keys into registers.  Slots outside the row hold key 0, which is below the key of
    // every finite score.
    const bool has_head = tid < nhead;
    const uint32_t khead = has_head ? order_key(seq[c0 + tid]) : 0u;
    const float *qbase = seq + c0 + nhead;                       // 16-byte aligned (unpooled)
    uint32_t key[QPT][4];
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
    for (int i = 0; i < QPT; ++i) {
        const int xw = 4 * (i * kSelThreads + 64 * wave_u);      // the wave's first index of this step
        if constexpr (POOL) {
            const int x0 = xw + 4 * lane;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                key[i][j] = (x0 + j < nq_el)
                    ? order_key(pooled_score(seq, nk, c0 + x0 + j, p.pool_r, p.pool_mode, p.pool_inv)) : 0u;
        } else if (xw + 255 < nq_el) {                           // all of its 64 quads lie inside the row
            const float4 t = *(const float4 *)(qbase + xw + 4 * lane);
            key[i][0] = order_key(t.x);  key[i][1] = order_key(t.y);
            key[i][2] = order_key(t.z);  key[i][3] = order_key(t.w);
        } else {
            const int x0 = xw + 4 * lane;
#pragma unroll
            for (int j = 0; j < 4; ++j) key[i][j] = (x0 + j < nq_el) ? order_key(qbase[x0 + j]) : 0u;
        }
    }
    // row range over the real keys: an empty slot (key 0) wraps to the largest value under key - 1
    // and so never is the minimum
    uint32_t kmin = khead - 1u, kmax = khead;
#pragma unroll
    for (int i = 0; i < QPT; ++i) {
        kmin = min(kmin, min(min(key[i][0] - 1u, key[i][1] - 1u), min(key[i][2] - 1u, key[i][3] - 1u)));
        kmax = max(kmax, max(max(key[i][0], key[i][1]), max(key[i][2], key[i][3])));
    }
    wave_min_max(kmin, kmax);
    if (lane == 63) { wave_min[wave] = kmin; wave_max[wave] = kmax; }
    if (tid < kSelMaxProbes) probe_tot[tid] = 0;
    if (tid < kSelFinish + 4) fin_keys[tid] = 0;
    if (tid == 0) fin_count = 0;
    __syncthreads();
    kmin = wave_min[0];  kmax = wave_max[0];
#pragma unroll
    for (int w = 1; w < kSelWaves; ++w) { kmin = min(kmin, wave_min[w]); kmax = max(kmax, wave_max[w]); }
    kmin += 1u;                                                  // back from key - 1 (kk >= 1: the row has a real key)

    // ---- threshold search: largest T in [kmin, kmax] with count(key >= T) >= kk, by probes on the
    // key value with the bracket [lo, hi] and the two counts c_lo = count(key >= lo) >= kk >
    // c_above = count(key > hi) (see next_probe).  Every probed value is > lo >= kmin > 0, so empty
    // slots never count.  The waves' counts of a probe meet in an LDS counter of their own (integer
    // atomics; one fresh counter per probe, so none is ever cleared), which every thread reads
    // back after the barrier.  Once at most kSelFinish keys are left inside the bracket they are
    // collected in LDS (in any order) and one wave ranks them directly.
    uint32_t lo = kmin, hi = kmax;
    uint32_t c_lo = (uint32_t)n, c_above = 0;
    bool interp = true;
    int probe = 0;
    while (lo < hi && c_lo - c_above > (uint32_t)kSelFinish) {
        const uint32_t inside = c_lo - c_above;
        const uint32_t mid = next_probe(lo, hi, inside, (uint32_t)kk - c_above, interp);
        // Half of the comparisons are counted with a ballot and a scalar population count, half per
        // lane on the vector unit with one wave sum at the end.  The 16 waves of the workgroup (and
        // a second workgroup on the same compute unit) share one scalar unit: all on it, the probe
        // queues there (1.87 TB/s over 512 rows of 32768); all on the vector unit is slower again
        // (2.17 TB/s); the split reaches 2.29 TB/s.
        uint32_t c = (uint32_t)__popcll(__ballot(khead >= mid));
        uint32_t cl[2] = {0u, 0u};
#pragma unroll
        for (int i = 0; i < QPT; ++i) {
            c += (uint32_t)__popcll(__ballot(key[i][0] >= mid));
            c += (uint32_t)__popcll(__ballot(key[i][1] >= mid));
            cl[0] += key[i][2] >= mid ? 1u : 0u;
            cl[1] += key[i][3] >= mid ? 1u : 0u;
        }
        c += (uint32_t)__builtin_amdgcn_readlane((int)wave_incl_scan(cl[0] + cl[1]), 63);
        if (lane == 0) atomicAdd(&probe_tot[probe], c);
        __syncthreads();
        const uint32_t tot = probe_tot[probe];
        ++probe;
        if (tot >= (uint32_t)kk) { lo = mid; c_lo = tot; }
        else { hi = mid - 1u; c_above = tot; }
        interp = !interp || 4u * (c_lo - c_above) <= inside;
    }
    if (lo < hi) {
        // at most kSelFinish keys lie in [lo, hi] (empty slots, key 0 < lo, fall outside by the
        // unsigned wrap): the (kk - c_above)-th largest of them is T
        const uint32_t width = hi - lo;
        if (khead - lo <= width) fin_keys[atomicAdd(&fin_count, 1u)] = khead;
#pragma unroll
        for (int i = 0; i < QPT; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (key[i][j] - lo <= width) fin_keys[atomicAdd(&fin_count, 1u)] = key[i][j];
        __syncthreads();
        if (wave == 0) {
            const int m = (int)fin_count;                                 // <= kSelFinish = 64
            const uint32_t mine_k = lane < m ? fin_keys[lane] : 0u;
            uint32_t gt = 0, ge = 0;
            for (int j0 = 0; j0 < m; j0 += 4) {                           // slots past m hold 0: below every key
                const uint4 o4 = *(const uint4 *)(fin_keys + j0);
                const uint32_t o[4] = {o4.x, o4.y, o4.z, o4.w};
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    gt += o[x] > mine_k ? 1u : 0u;
                    ge += o[x] >= mine_k ? 1u : 0u;
                }
            }
            const uint32_t r = (uint32_t)kk - c_above;                    // 1 <= r <= m
            const bool hit = lane < m && gt < r && r <= ge;               // every hit lane holds the same key
            const uint64_t hb = __ballot(hit);
            if (hb != 0 && lane == (int)__builtin_ctzll(hb)) { fin_T = mine_k; fin_above = c_above + gt; }
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
    uint32_t pre[QPT];                      // prefix inside the wave, packed gt | eq << 16
#pragma unroll
    for (int i = 0; i < QPT; ++i) {
        uint32_t c = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {                  // empty slots hold key 0 < kmin <= T
            c += key[i][j] > T ? 1u : 0u;
            c += key[i][j] == T ? 0x10000u : 0u;
        }
        pre[i] = c;
    }
    {
        uint32_t incl[QPT];
#pragma unroll
        for (int i = 0; i < QPT; ++i) incl[i] = pre[i];
        wave_incl_scan_n(incl);
#pragma unroll
        for (int i = 0; i < QPT; ++i) {
            pre[i] = incl[i] - pre[i];                 // exclusive
            if (lane == 63) cnt[i * kSelWaves + wave] = incl[i];
        }
    }
    __syncthreads();
    // every wave scans the (step, wave) totals itself (at most 128 of them, two per lane) and picks
    // the offsets of its own QPT steps: no further barrier
    constexpr int NC = kSelWaves * QPT;
    uint32_t step_off[QPT];                 // keys > T | == T << 16 before this wave's part of step i
    uint32_t eq_total;
    {
        uint32_t v[2] = {lane < NC ? cnt[lane] : 0u, 64 + lane < NC ? cnt[64 + lane] : 0u};
        uint32_t sc[2] = {v[0], v[1]};
        wave_incl_scan_n(sc);
        const uint32_t tot0 = (uint32_t)__builtin_amdgcn_readlane((int)sc[0], 63);
        const uint32_t ex0 = sc[0] - v[0] + head_tot, ex1 = sc[1] - v[1] + tot0 + head_tot;
#pragma unroll
        for (int i = 0; i < QPT; ++i) {
            const int e = i * kSelWaves + wave_u;
            step_off[i] = e < 64 ? (uint32_t)__builtin_amdgcn_readlane((int)ex0, e)
                                 : (uint32_t)__builtin_amdgcn_readlane((int)ex1, e - 64);
        }
        eq_total = (head_tot + tot0 + (uint32_t)__builtin_amdgcn_readlane((int)sc[1], 63)) >> 16;
    }

    // ---- stable compaction
    if (has_head) {
        const int gt_before = (int)(pre_head & 0xffffu), eq_before = (int)(pre_head >> 16);
        const bool sel = khead > T || (khead == T && eq_before < krem);
        if (sel) out[gt_before + min(eq_before, krem)] = c0 + tid;
        if (mrow) mrow[c0 + tid] = sel ? 1 : 0;
    }
    // Common case: every key equal to T is kept (no tie is cut, e.g. T is unique).  A key is then
    // selected iff it is >= T and its slot is the count of such keys before it.
    const bool ties_all_kept = (int)eq_total <= krem;
    // the quads' mask bytes go out as one 4-byte store where the mask tensor is aligned like that
    const bool mask_dwords = mrow && (((uint32_t)(uintptr_t)(mrow + c0 + nhead)) & 3u) == 0;
    // The comparisons of the counting pass are made again here, against a copy of T the compiler
    // cannot relate to the first: kept alive across the scans, their 64 lane masks per wave do not
    // fit the scalar registers and are spilled lane by lane.
    uint32_t Tc = T;
    asm volatile("" : "+v"(Tc));
#pragma unroll
    for (int i = 0; i < QPT; ++i) {
        const int x0 = 4 * (i * kSelThreads + tid);
        const uint32_t before = step_off[i] + pre[i];
        uint32_t mbytes = 0;
        if (ties_all_kept) {
            int pos = (int)(before & 0xffffu) + (int)(before >> 16);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool sel = key[i][j] >= Tc;                             // never true for an empty slot
                if (sel) out[pos] = c0 + nhead + x0 + j;
                pos += sel ? 1 : 0;
                mbytes |= sel ? (1u << (8 * j)) : 0u;
            }
        } else {
            int gt_before = (int)(before & 0xffffu), eq_before = (int)(before >> 16);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool is_gt = key[i][j] > Tc, is_eq = key[i][j] == Tc;
                const bool sel = is_gt || (is_eq && eq_before < krem);
                if (sel) out[gt_before + min(eq_before, krem)] = c0 + nhead + x0 + j;
                gt_before += is_gt ? 1 : 0;
                eq_before += is_eq ? 1 : 0;
                mbytes |= sel ? (1u << (8 * j)) : 0u;
            }
        }
        if (mrow && x0 < nq_el) {
            uint8_t *mp = mrow + c0 + nhead + x0;
            if (mask_dwords && x0 + 3 < nq_el) *(uint32_t *)mp = mbytes;
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
