// Causal / GQA / ragged prefill attention for gfx950 (flash-style forward).
//
// Computes, per sequence b, query head h (KV head g = h / G) and query i,
//   S[i,j] = s <q_i, k_j>  for j <= i + delta_b,   lse = ln sum_j exp S[i,j],
//   o_i = sum_j exp(S[i,j] - lse) v_j
// (paper Section 2.2.3, scaled dot-product attention; the mask is the
// autoregressive one, aligned bottom-right so a chunk of new queries sees the
// whole KV prefix, Section 3.3 "LLM Engine", chunked prefill).
//
// Work decomposition
//   workgroup = NWAVES wavefronts, each owning 32 consecutive queries of one
//   (sequence, query head); key/value tiles of 64 keys stream through LDS
//   (double buffered, register-staged prefetch of the next tile).
//   Per 32-key block a wave computes S^T = K Q^T with v_mfma_f32_32x32x16_bf16
//   (A = K rows from LDS, B = Q fragments held in registers), so lane l owns
//   query (l % 32) and the 16 accumulator registers hold 16 different keys:
//   row max / row sum are in-lane reductions plus one exchange between lanes
//   l and l+32.  O^T = V^T P^T reuses those registers directly as the B
//   operand (the contraction index "key" may be permuted freely as long as V^T
//   is stored with the same permutation in LDS).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pdd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) float f32x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

struct AttnParams {
    const uint16_t *q, *k, *v;
    uint16_t *o;
    float *lse;
    const int32_t *cu_q, *cu_k;
    int64_t q_st, q_sh, k_st, k_sh, v_st, v_sh, o_st, o_sh;
    int32_t B, Hq, Hkv, G, total_q, total_k, n_qtiles;
    float scale_log2;  // softmax scale * log2(e)
    // Only read by kernels built with the importance sweep: partial column sums
    // [G * n_qtiles][Hkv][total_k], slice hg * n_qtiles + t written by the workgroup of query
    // head g * G + hg and query tile t (every key of its sequence, zeros included).
    float *imp_part;
};

constexpr int kBN = 64;  // keys per LDS tile

template <int D>
struct AttnSmem {
    static constexpr int KSTR = D + 8;    // bf16 elements per K row (16 B pad)
    static constexpr int VSTR = kBN + 8;  // bf16 elements per V^T row
    static constexpr int K_ELEMS = kBN * KSTR;
    static constexpr int V_ELEMS = D * VSTR;
    static constexpr int BYTES = 2 * (K_ELEMS + V_ELEMS) * 2;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float max3(float a, float b, float c)
{
    // Compiles to one v_max3_f32.  Deliberately not inline assembly: the operands are MFMA
    // results, and only for instructions it knows does the compiler insert the wait states
    // the hardware needs between an MFMA writing a register and a VALU instruction reading it
    // (an assembly v_max3 right behind the MFMA reads the accumulator before the last pass
    // has written it, which made the running max, and with it the rounding, depend on timing).
    return fmaxf(fmaxf(a, b), c);
}

__device__ __forceinline__ float xchg_half(float x)
{
    // value held by the lane 32 positions away (v_permlane32_swap: one VALU op, no LDS)
    const uint32_t u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

template <int D, int NWAVES>
__global__ __launch_bounds__(NWAVES * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_fwd_kernel(const AttnParams p)
{
    using SM = AttnSmem<D>;
    constexpr int NT = NWAVES * 64;
    constexpr int BM = NWAVES * 32;
    constexpr int KCH = D / 8;                       // 16-byte chunks per K row
    constexpr int K_PASSES = (kBN * KCH + NT - 1) / NT;
    constexpr int V_TASKS = (kBN / 4) * (D / 4);     // 4 keys x 4 dims each
    constexpr int V_PASSES = (V_TASKS + NT - 1) / NT;
    constexpr int NKK = D / 16;                      // MFMA k-steps for QK^T
    constexpr int NDB = D / 32;                      // 32-row blocks of O^T

    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t *Ks = smem;                       // [2][K_ELEMS]
    uint16_t *Vs = smem + 2 * SM::K_ELEMS;     // [2][V_ELEMS]

    // ---- block -> (kv head g fastest, head-in-group, sequence, q tile heavy first)
    int bid = blockIdx.x;
    const int g = bid % p.Hkv;  bid /= p.Hkv;
    const int hg = bid % p.G;   bid /= p.G;
    const int b = bid % p.B;    bid /= p.B;
    const int t = p.n_qtiles - 1 - bid;
    const int h = g * p.G + hg;

    const int qs = min(p.cu_q[b], p.total_q), qe = min(p.cu_q[b + 1], p.total_q);
    const int ks = min(p.cu_k[b], p.total_k), ke = min(p.cu_k[b + 1], p.total_k);
    const int nq = qe - qs, nk = ke - ks;
    const int m0 = t * BM;
    if (m0 >= nq || nq <= 0) return;
    const int delta = nk - nq;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, hh = lane >> 5;

    const int wave_q0 = m0 + 32 * wave;              // first query of this wave
    const int qrow = wave_q0 + n;
    const int qrow_c = min(qrow, nq - 1);
    const int lim = qrow_c + delta;                  // last visible key of this lane's query
    const int wave_lim_max = min(wave_q0 + 31, nq - 1) + delta;
    const int wave_lim_min = min(wave_q0, nq - 1) + delta;

    // keys needed by the workgroup: [0, kend)
    const int kend = min(nk, min(m0 + BM, nq) + delta);
    const int n_tiles = kend > 0 ? (kend + kBN - 1) / kBN : 0;

    // ---- Q fragments (B operand): query n, dims 16*kk + 8*hh .. +7
    bf16x8 qf[NKK];
    {
        const uint16_t *qp = p.q + (int64_t)(qs + qrow_c) * p.q_st + (int64_t)h * p.q_sh + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) qf[kk] = *(const bf16x8 *)(qp + 16 * kk);
    }

    const uint16_t *kbase = p.k + (int64_t)ks * p.k_st + (int64_t)g * p.k_sh;
    const uint16_t *vbase = p.v + (int64_t)ks * p.v_st + (int64_t)g * p.v_sh;

    u32x4 kreg[K_PASSES];
    u32x2 vreg[V_PASSES][4];

    auto load_tile = [&](int it) {
        const int j0 = it * kBN;
#pragma unroll
        for (int ps = 0; ps < K_PASSES; ++ps) {
            const int c = tid + ps * NT;
            if (K_PASSES * NT == kBN * KCH || c < kBN * KCH) {
                const int key = min(j0 + c / KCH, nk - 1);
                kreg[ps] = *(const u32x4 *)(kbase + (int64_t)key * p.k_st + (c % KCH) * 8);
            }
        }
#pragma unroll
        for (int ps = 0; ps < V_PASSES; ++ps) {
            const int task = tid + ps * NT;
            if (V_PASSES * NT == V_TASKS || task < V_TASKS) {
                const int dg = task % (D / 4), kg = task / (D / 4);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int key = min(j0 + 4 * kg + i, nk - 1);
                    vreg[ps][i] = *(const u32x2 *)(vbase + (int64_t)key * p.v_st + 4 * dg);
                }
            }
        }
    };

    auto store_tile = [&](int buf) {
        uint16_t *Kb = Ks + buf * SM::K_ELEMS;
        uint16_t *Vb = Vs + buf * SM::V_ELEMS;
#pragma unroll
        for (int ps = 0; ps < K_PASSES; ++ps) {
            const int c = tid + ps * NT;
            if (K_PASSES * NT == kBN * KCH || c < kBN * KCH)
                *(u32x4 *)(Kb + (c / KCH) * SM::KSTR + (c % KCH) * 8) = kreg[ps];
        }
#pragma unroll
        for (int ps = 0; ps < V_PASSES; ++ps) {
            const int task = tid + ps * NT;
            if (V_PASSES * NT == V_TASKS || task < V_TASKS) {
                const int dg = task % (D / 4), kg = task / (D / 4);
                // quad of 4 keys -> slot inside its 16-key group: (0,1,2,3) -> (0,2,1,3)
                const int qd = kg & 3;
                const int slot = 16 * (kg >> 2) + 4 * (((qd & 1) << 1) | (qd >> 1));
                const u32x2 r0 = vreg[ps][0], r1 = vreg[ps][1], r2 = vreg[ps][2], r3 = vreg[ps][3];
                // 4x4 transpose of 16-bit values: row = key, column = dim
                u32x2 c0, c1, c2, c3;
                c0.x = (r0.x & 0xffffu) | (r1.x << 16);  c0.y = (r2.x & 0xffffu) | (r3.x << 16);
                c1.x = (r0.x >> 16) | (r1.x & 0xffff0000u);  c1.y = (r2.x >> 16) | (r3.x & 0xffff0000u);
                c2.x = (r0.y & 0xffffu) | (r1.y << 16);  c2.y = (r2.y & 0xffffu) | (r3.y << 16);
                c3.x = (r0.y >> 16) | (r1.y & 0xffff0000u);  c3.y = (r2.y >> 16) | (r3.y & 0xffff0000u);
                uint16_t *dst = Vb + (4 * dg) * SM::VSTR + slot;
                *(u32x2 *)(dst) = c0;
                *(u32x2 *)(dst + SM::VSTR) = c1;
                *(u32x2 *)(dst + 2 * SM::VSTR) = c2;
                *(u32x2 *)(dst + 3 * SM::VSTR) = c3;
            }
        }
    };

    f32x16 oacc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[db][e] = 0.f;
    float m_run = -INFINITY;   // running max of raw (unscaled) scores, shared by both halves
    float l_run = 0.f;         // this half's partial row sum
    const float c2 = p.scale_log2;

    if (n_tiles > 0) {
        load_tile(0);
        store_tile(0);
    }
    __syncthreads();
    // Everything loaded so far (Q fragments included) has landed: say so, or the
    // compiler re-waits for the Q loads inside the loop, behind the prefetches.
    __builtin_amdgcn_s_waitcnt(0);

    for (int it = 0; it < n_tiles; ++it) {
        const int buf = it & 1;
        const int j0 = it * kBN;
        const bool more = it + 1 < n_tiles;
        if (more) load_tile(it + 1);

        if (j0 <= wave_lim_max) {   // wave-uniform: some query of this wave sees this tile
            const uint16_t *Kb = Ks + buf * SM::K_ELEMS;
            const uint16_t *Vb = Vs + buf * SM::V_ELEMS;
            const bool blk1 = (j0 + 32 <= wave_lim_max);   // second 32-key block visible?

            f32x16 s0, s1;
#pragma unroll
            for (int e = 0; e < 16; ++e) { s0[e] = 0.f; s1[e] = 0.f; }
            {
                const uint16_t *ka = Kb + n * SM::KSTR + 8 * hh;
#pragma unroll
                for (int kk = 0; kk < NKK; ++kk) {
                    const bf16x8 a = *(const bf16x8 *)(ka + 16 * kk);
                    s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s0, 0, 0, 0);
                }
                if (blk1) {
#pragma unroll
                    for (int kk = 0; kk < NKK; ++kk) {
                        const bf16x8 a = *(const bf16x8 *)(ka + 32 * SM::KSTR + 16 * kk);
                        s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s1, 0, 0, 0);
                    }
                }
            }
            // ---- causal / length mask (only tiles that touch the diagonal)
            if (j0 + kBN - 1 > wave_lim_min) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int j = j0 + 8 * (e >> 2) + 4 * hh + (e & 3);
                    if (j > lim) s0[e] = -INFINITY;
                    if (j + 32 > lim) s1[e] = -INFINITY;
                }
            }
            // ---- online softmax
            float tmax = max3(s0[0], s0[1], s0[2]);
#pragma unroll
            for (int e = 3; e < 15; e += 2) tmax = max3(tmax, s0[e], s0[e + 1]);
#pragma unroll
            for (int e = 0; e < 16; e += 2) tmax = max3(tmax, s1[e], s1[e + 1]);
            tmax = max3(tmax, s0[15], xchg_half(max3(tmax, s0[15], s0[15])));
            const float m_new = fmaxf(m_run, tmax);
            if (__any(m_new > m_run)) {           // wave-uniform: rescale only when a max moved
                const float alpha = (m_run == -INFINITY) ? 0.f : fast_exp2((m_run - m_new) * c2);
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < NDB; ++db)
#pragma unroll
                    for (int e = 0; e < 16; ++e) oacc[db][e] *= alpha;
                m_run = m_new;
            }
            const float mc = (m_run == -INFINITY) ? 0.f : m_run * c2;
            float psum = 0.f;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                s0[e] = fast_exp2(fmaf(s0[e], c2, -mc));
                psum += s0[e];
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                s1[e] = fast_exp2(fmaf(s1[e], c2, -mc));
                psum += s1[e];
            }
            l_run += psum;

            // ---- O^T += V^T P^T ; 16 keys per step, B operand straight from s0/s1
            const uint16_t *va = Vb + n * SM::VSTR + 8 * hh;
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                if (st >= 2 && !blk1) break;
                f32x8 pf;
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[e] = (st < 2) ? s0[8 * (st & 1) + e] : s1[8 * (st & 1) + e];
                const bf16x8 pb = __builtin_convertvector(pf, bf16x8);
#pragma unroll
                for (int db = 0; db < NDB; ++db) {
                    const bf16x8 a = *(const bf16x8 *)(va + (32 * db) * SM::VSTR + 16 * st);
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, oacc[db], 0, 0, 0);
                }
            }
        }

        if (more) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: normalise, write O (bf16) and LSE (fp32, natural log)
    const float l_tot = l_run + xchg_half(l_run);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (qrow < nq) {
        uint16_t *op = p.o + (int64_t)(qs + qrow) * p.o_st + (int64_t)h * p.o_sh;
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
#pragma unroll
            for (int bq = 0; bq < 4; ++bq) {
                f32x4 x;
#pragma unroll
                for (int r = 0; r < 4; ++r) x[r] = oacc[db][4 * bq + r] * inv;
                const bf16x4 y = __builtin_convertvector(x, bf16x4);
                *(bf16x4 *)(op + 32 * db + 8 * bq + 4 * hh) = y;
            }
        }
        if (hh == 0) {
            const float lse = l_tot > 0.f
                ? (m_run * c2 + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f
                : -INFINITY;
            p.lse[(int64_t)h * p.total_q + qs + qrow] = lse;
        }
    }
}

}  // namespace pdd
