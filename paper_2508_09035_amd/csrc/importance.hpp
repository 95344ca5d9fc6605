// Token importance from the observation window (paper Section 3.2, "Prompt
// Refiner": the normalised attention weight of the last segment of queries
// against the entire K, summed along the query dimension).
//
//   imp[g, j] = sum_{h in group g} sum_{i in window, i + delta >= j}
//               exp(s <q_i, k_j> - lse[h, i])
//
// The final log-sum-exp of every window row is an input, so each probability
// is recomputed from one QK^T tile and added into a per-key column sum; the
// attention matrix is never stored.  Work is split over KEYS: a workgroup of 4
// waves owns 256 keys, each wave 64 of them (two 32-key groups whose K
// fragments stay in registers as B operands for the whole kernel); with KG = 1
// it owns 128 keys, one 32-key group per wave, which small launches prefer.  The window
// rows of the G query heads are streamed through LDS in blocks of 32 rows
// (buffer_load ... lds, double buffered, swizzled like the attention K tile)
// together with their log-sum-exp values (four buffers, three blocks in flight:
// with little arithmetic per block the kernel lives on hiding the load latency),
// so every Q fragment read from LDS feeds KG MFMAs and every Q row is fetched
// from L2 once per workgroup.
// S = Q K^T puts key (l % 32) in lane l and 16 query rows in its accumulator
// registers, so the sum over queries is in-lane; no atomics, fixed summation
// order, deterministic.
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
    // Row split: the window rows of a workgroup's keys are divided over n_split workgroups; with
    // n_split > 1 workgroup r writes its partial column sums to part[r][Hkv][total_k] (every
    // element of a sequence, zeros included) and importance_reduce_kernel adds them in the
    // fixed order r = 0, 1, ...
    int32_t n_split;
    float *part;
};

constexpr int kImpWaves = 4;
constexpr int kImpBK = 64 * kImpWaves;  // keys per workgroup
constexpr int kImpBufs = 4;             // LDS ring of query-row blocks
constexpr int kImpAhead = 3;            // blocks in flight

// 4 bytes per lane from the buffer into LDS at lds_addr + 4 * lane (see dma16_to_lds)
__device__ __forceinline__ void dma4_to_lds(i32x4 rsrc, uint32_t lds_addr, uint32_t voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc)
                 : "memory", "m0");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

template <int D, int KG = 2>
__global__ __launch_bounds__(kImpWaves * 64) __attribute__((amdgpu_waves_per_eu(3, 4)))
void importance_kernel(const ImpParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int NKK = D / 16;
    constexpr int ROW_BYTES = D * 2;             // one Q row in LDS
    constexpr int CH = D / 8;                    // 16-byte chunks per row
    constexpr int QBLK_BYTES = 32 * ROW_BYTES;   // one block of 32 query rows
    constexpr int NLD = QBLK_BYTES / (kImpWaves * 1024);   // DMA instructions per block per wave (2 or 1)
    constexpr int PER_ITEM = NLD + 1;            // DMA instructions per block per wave (Q rows + LSE)
    __shared__ __attribute__((aligned(1024))) uint8_t qs_lds[kImpBufs][QBLK_BYTES];
    __shared__ __attribute__((aligned(256))) float lse_lds[kImpBufs][kImpWaves][64];   // a private copy per wave

    int bid = blockIdx.x;
    const int g = bid % p.Hkv;  bid /= p.Hkv;
    const int b = bid % p.B;    bid /= p.B;
    const int kt = bid % p.n_ktiles;
    const int split = bid / p.n_ktiles;

    const int qs = min(p.cu_q[b], p.total_q), qe = min(p.cu_q[b + 1], p.total_q);
    const int ks = min(p.cu_k[b], p.total_k), ke = min(p.cu_k[b + 1], p.total_k);
    const int nq = qe - qs, nk = ke - ks;
    constexpr int WKEYS = 32 * KG;               // keys per wave
    const int j_wg0 = kt * (WKEYS * kImpWaves);
    if (j_wg0 >= nk) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, hh = lane >> 5;
    const int delta = nk - nq;
    const int W = (p.window < 0 || p.window > nq) ? nq : p.window;
    const int iw0 = nq - W;                       // first window row
    const int jw0 = j_wg0 + WKEYS * wave;         // first key of this wave

    // K fragments (B operand) of the wave's KG 32-key groups: key j, dims 16 kk + 8 hh .. +7
    bf16x8 kf[KG][NKK];
    int jkey[KG];
#pragma unroll
    for (int kg = 0; kg < KG; ++kg) {
        jkey[kg] = jw0 + 32 * kg + n;
        const uint16_t *kp = p.k + (int64_t)(ks + min(jkey[kg], nk - 1)) * p.k_st + (int64_t)g * p.k_sh + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) kf[kg][kk] = *(const bf16x8 *)(kp + 16 * kk);
    }
    const float c2 = p.scale_log2;
    constexpr float kLog2e = 1.4426950408889634f;
    float colsum[KG] = {};

    if (nq > 0 && delta >= 0 && W > 0) {
        // row blocks: (head in group, 32-row block of the window); blocks whose rows all lie
        // before key j_wg0 - delta see none of this workgroup's keys and are skipped
        const int n_rb = (W + 31) / 32;
        const int rb_first = min(n_rb, max(0, (j_wg0 - delta - iw0) / 32));
        const int n_items_all = p.G * (n_rb - rb_first);
        // this workgroup's share of the row blocks: items [item0, item0 + n_items)
        const int per_split = (n_items_all + p.n_split - 1) / p.n_split;
        const int item0 = min(split * per_split, n_items_all);
        const int n_items = min(per_split, n_items_all - item0);

        // Q rows of this sequence, all heads: buffer descriptor spanning the whole sequence
        const uint16_t *qbase = p.q + (int64_t)qs * p.q_st;
        const uint32_t q_row_bytes = (uint32_t)p.q_st * 2u;
        const uint32_t q_span = (uint32_t)(nq - 1) * q_row_bytes + (uint32_t)p.Hq * (uint32_t)p.q_sh * 2u;
        const i32x4 rsQ = make_rsrc(qbase, q_span);
        const i32x4 rsL = make_rsrc(p.lse, (uint32_t)p.Hq * (uint32_t)p.total_q * 4u);
        const uint32_t q_lds = lds_addr_of(&qs_lds[0][0]);
        const uint32_t l_lds = lds_addr_of(&lse_lds[0][wave][0]);
        // lane -> (row in block, chunk position); LDS chunk position holds chunk pos ^ swizzle(row)
        uint32_t qvoff[NLD];
        int qrow_l[NLD];
#pragma unroll
        for (int ci = 0; ci < NLD; ++ci) {
            const int flat = (wave + kImpWaves * ci) * 64 + lane;          // 16-byte slot in the block
            const int r = flat / CH, pos = flat % CH;
            const int c = D == 128 ? (pos ^ swz_row<128>(r)) : (pos ^ ((r >> 1) & 7));
            qrow_l[ci] = r;
            qvoff[ci] = (uint32_t)c * 16u;
        }
        // Blocks are requested and worked on in order, so the (head, row block) pair of the next
        // request and the row block in work are counted along: one division here, none per block.
        const int n_rbs = n_rb - rb_first;           // row blocks per head that this workgroup walks
        int iss_hg = n_rbs > 0 ? item0 / n_rbs : 0, iss_rb = n_rbs > 0 ? item0 % n_rbs : 0;
        int cur_rb = iss_rb;
        auto issue_item = [&](int buf) {              // the next block in order
            const int h = g * p.G + iss_hg;
            const int i0 = iw0 + 32 * (rb_first + iss_rb);
            if (++iss_rb == n_rbs) { iss_rb = 0; ++iss_hg; }
#pragma unroll
            for (int ci = 0; ci < NLD; ++ci) {
                const int i = min(i0 + qrow_l[ci], nq - 1);
                dma16_to_lds(rsQ, q_lds + buf * QBLK_BYTES + 1024 * (wave + kImpWaves * ci),
                             (uint32_t)i * q_row_bytes + (uint32_t)h * (uint32_t)p.q_sh * 2u + qvoff[ci]);
            }
            const int il = min(i0 + (lane & 31), nq - 1);
            dma4_to_lds(rsL, l_lds + buf * (kImpWaves * 256), ((uint32_t)h * (uint32_t)p.total_q + (uint32_t)(qs + il)) * 4u);
        };
        // A-operand read address of row n, chunk 2 kk + hh
        uint32_t qaddr[NKK];
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
            const int c = 2 * kk + hh;
            const int cs = D == 128 ? (c ^ swz_row<128>(n)) : (c ^ ((n >> 1) & 7));
            qaddr[kk] = (uint32_t)n * ROW_BYTES + (uint32_t)cs * 16u;
        }

        // The first row blocks are requested while the K fragment loads are still in flight; one
        // wait then ends both (the blocks were requested together and land together).  With the K
        // loads done here the compiler places no load waits inside the loop, where they would also
        // wait for the asynchronous row-block transfers in flight.
        for (int i = 0; i < kImpAhead && i < n_items; ++i) issue_item(i);
        __builtin_amdgcn_s_waitcnt(0);
        for (int item = 0; item < n_items; ++item) {
            const int buf = item & (kImpBufs - 1);
            // this block's loads are done once at most the blocks issued after it are outstanding
            const int newer = min(kImpAhead - 1, n_items - 1 - item);
            if (newer == 2) wait_vmcnt<2 * PER_ITEM>();
            else if (newer == 1) wait_vmcnt<PER_ITEM>();
            else wait_vmcnt<0>();
            __syncthreads();     // every wave's part of the block has landed; the buffer refilled below is free
            if (item + kImpAhead < n_items) issue_item((item + kImpAhead) & (kImpBufs - 1));
            const int i0 = iw0 + 32 * (rb_first + cur_rb);
            if (++cur_rb == n_rbs) cur_rb = 0;
            const int i_last = min(i0 + 31, nq - 1);
            if (jw0 <= i_last + delta && jw0 < nk) {       // some row of the block sees some key of the wave
                const uint8_t *qb = &qs_lds[buf][0];
                f32x16 sc[KG];
                const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < NKK; ++kk) {
                    const bf16x8 a = *(const bf16x8 *)(qb + qaddr[kk]);
#pragma unroll
                    for (int kg = 0; kg < KG; ++kg)
                        sc[kg] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, kf[kg][kk], kk == 0 ? zero16 : sc[kg], 0, 0, 0);
                }
                // log2-domain LSE of rows 8 (e/4) + 4 hh + (e%4)
                f32x4 l2[4];
#pragma unroll
                for (int bq = 0; bq < 4; ++bq) l2[bq] = *(const f32x4 *)&lse_lds[buf][wave][8 * bq + 4 * hh] * kLog2e;
                // rows beyond the sequence end or keys beyond a row's reach contribute nothing
                const bool partial = (i0 + 31 > nq - 1) || (jw0 + WKEYS - 1 > i0 + delta) || (jw0 + WKEYS - 1 > nk - 1);
                if (!partial) {
#pragma unroll
                    for (int e = 0; e < 16; ++e)
#pragma unroll
                        for (int kg = 0; kg < KG; ++kg)
                            colsum[kg] += fast_exp2(fmaf(sc[kg][e], c2, -l2[e >> 2][e & 3]));
                } else {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int i = i0 + 8 * (e >> 2) + 4 * hh + (e & 3);
#pragma unroll
                        for (int kg = 0; kg < KG; ++kg) {
                            const float pe = fast_exp2(fmaf(sc[kg][e], c2, -l2[e >> 2][e & 3]));
                            colsum[kg] += (i < nq && jkey[kg] <= i + delta && jkey[kg] < nk) ? pe : 0.f;
                        }
                    }
                }
            }
        }
    }
#pragma unroll
    for (int kg = 0; kg < KG; ++kg) {
        const float tot = colsum[kg] + xchg_half(colsum[kg]);
        float *dst = p.n_split > 1 ? p.part + (int64_t)split * p.Hkv * p.total_k : p.imp;
        if (hh == 0 && jkey[kg] < nk) dst[(int64_t)g * p.total_k + ks + jkey[kg]] = tot;
    }
#else
    (void)p;
#endif
}

// imp[x] = part[0][x] + part[1][x] + ... in that order, x over Hkv * total_k elements
__global__ __launch_bounds__(256) void importance_reduce_kernel(const float *part, float *imp, int64_t n, int n_split)
{
    const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (x >= n) return;
    float acc = part[x];
    for (int r = 1; r < n_split; ++r) acc += part[(int64_t)r * n + x];
    imp[x] = acc;
}

}  // namespace pdd
