// Causal / GQA / ragged prefill attention, head_dim 128: 64 queries per wavefront.
//
// Same mathematics, LDS layout and register layout as attn_fwd_d128.hpp.  What
// changes is the work per wave: a wave owns TWO groups of 32 queries ("a" and
// "b") and one wave runs per SIMD with the full 512-register budget.
//   * every K / V^T fragment read from LDS feeds two MFMAs (one per group),
//     which halves the LDS fragment traffic per flop -- the resource that
//     limited the 32-queries-per-wave kernel;
//   * the two groups alternate inside one instruction stream: while the matrix
//     pipe runs QK^T(u+1) and PV(u) of one group, the vector ALU computes the
//     exponentials of the other group.  No second wave is needed to hide the
//     softmax arithmetic.
// Workgroup = 4 waves = 256 queries.  K/V tiles (64 keys) are triple buffered in
// LDS and filled with buffer_load ... lds; tile t+2 is requested at the start of
// tile iteration t and awaited, with one workgroup barrier, at its end.
#pragma once
#include "attn_fwd_d128.hpp"

namespace pdd {

constexpr int kW64Waves = 4;
constexpr int kW64BM = 64 * kW64Waves;

__global__ __launch_bounds__(kW64Waves * 64) __attribute__((amdgpu_waves_per_eu(1, 1)))
void attn_fwd_d128_w64_kernel(const AttnParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the body uses gfx950-only builtins; the host pass needs the stub only
    constexpr int NW = kW64Waves, BM = kW64BM;
    constexpr int NKK = 8, NDB = 4;
    constexpr int NLD = 16 / NW;          // LDS-DMA instructions per tile per wave

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem_w64[];
    uint8_t *Ks = smem_w64;                               // [3][kTileBytes], tile t in buffer t % 3
    uint8_t *Vs = smem_w64 + kAttn128Bufs * kTileBytes;   // [3][kTileBytes]

    int bid = blockIdx.x;
    const int g = bid % p.Hkv;  bid /= p.Hkv;
    const int hg = bid % p.G;   bid /= p.G;
    const int b = bid % p.B;    bid /= p.B;
    const int qt = p.n_qtiles - 1 - bid;                  // heaviest q tiles first
    const int h = g * p.G + hg;

    const int qs = min(p.cu_q[b], p.total_q), qe = min(p.cu_q[b + 1], p.total_q);
    const int ks = min(p.cu_k[b], p.total_k), ke = min(p.cu_k[b + 1], p.total_k);
    const int nq = qe - qs, nk = ke - ks;
    const int m0 = qt * BM;
    if (m0 >= nq || nq <= 0) return;
    const int delta = nk - nq;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, hh = lane >> 5;

    // per query group r (0 = a, 1 = b)
    int qrow[2], lim[2], grp_lim_max[2], grp_lim_min[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int q0 = m0 + 64 * wave + 32 * r;
        qrow[r] = q0 + n;
        lim[r] = min(qrow[r], nq - 1) + delta;            // last visible key of this lane's query
        grp_lim_max[r] = min(q0 + 31, nq - 1) + delta;
        grp_lim_min[r] = min(q0, nq - 1) + delta;
    }
    const int kend = min(nk, min(m0 + BM, nq) + delta);
    const int n_tiles = kend > 0 ? (kend + kBN - 1) / kBN : 0;

    // ---- Q fragments (B operand of S^T = K Q^T): query n of each group, dims 16 kk + 8 hh .. +7
    bf16x8 qf[2][NKK];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const uint16_t *qp = p.q + (int64_t)(qs + min(qrow[r], nq - 1)) * p.q_st + (int64_t)h * p.q_sh + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) qf[r][kk] = *(const bf16x8 *)(qp + 16 * kk);
    }

    // ---- K / V tiles: HBM -> LDS
    const uint16_t *kbase = p.k + (int64_t)ks * p.k_st + (int64_t)g * p.k_sh;
    const uint16_t *vbase = p.v + (int64_t)ks * p.v_st + (int64_t)g * p.v_sh;
    const uint32_t k_row_bytes = (uint32_t)p.k_st * 2u, v_row_bytes = (uint32_t)p.v_st * 2u;
    const uint32_t k_span = nk > 0 ? (uint32_t)(nk - 1) * k_row_bytes + 256u : 0u;
    const uint32_t v_span = nk > 0 ? (uint32_t)(nk - 1) * v_row_bytes + 256u : 0u;
    const i32x4 rsK = make_rsrc(kbase, k_span), rsV = make_rsrc(vbase, v_span);
    const uint32_t ks_lds = lds_addr_of(Ks), vs_lds = lds_addr_of(Vs);
    uint32_t kvoff[NLD], vvoff[NLD];
#pragma unroll
    for (int ci = 0; ci < NLD; ++ci) {
        const int r = 4 * (wave + NW * ci) + (lane >> 4);
        const int c = (lane & 15) ^ swz16(r);
        kvoff[ci] = (uint32_t)r * k_row_bytes + (uint32_t)c * 16u;
        vvoff[ci] = (uint32_t)r * v_row_bytes + (uint32_t)c * 16u;
    }
    auto issue_tile = [&](int tile) {     // K(tile) and V(tile) -> buffer tile % 3
        if (tile >= n_tiles) return;
        const uint32_t boff = (uint32_t)(tile % 3) * kTileBytes;
        const uint32_t ko = (uint32_t)tile * kBN * k_row_bytes, vo = (uint32_t)tile * kBN * v_row_bytes;
#pragma unroll
        for (int ci = 0; ci < NLD; ++ci)
            dma16_to_lds(rsK, ks_lds + boff + 1024 * (wave + NW * ci), kvoff[ci] + ko);
#pragma unroll
        for (int ci = 0; ci < NLD; ++ci)
            dma16_to_lds(rsV, vs_lds + boff + 1024 * (wave + NW * ci), vvoff[ci] + vo);
    };

    // ---- LDS fragment addresses (bytes inside a tile), see attn_fwd_d128.hpp
    uint32_t kaddr[NKK], vaddr[NDB][2];
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) kaddr[kk] = (uint32_t)n * 256u + (uint32_t)(((2 * kk + hh) ^ swz16(n)) * 16);
    {
        const int s16 = lane & 15, dhalf = (lane >> 4) & 1;
#pragma unroll
        for (int eg = 0; eg < 2; ++eg) {
            const int row = 8 * eg + 4 * hh + (s16 >> 2);
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                const int chunk = 4 * db + 2 * dhalf + ((s16 & 3) >> 1);
                vaddr[db][eg] = (uint32_t)row * 256u + (uint32_t)((chunk ^ swz16(row)) * 16) + 8u * (s16 & 1);
            }
        }
    }
    // byte offset of 32-key block u inside the K (V) buffers
    auto k_block_off = [&](int u) { return (uint32_t)((u >> 1) % 3) * kTileBytes + (uint32_t)(u & 1) * (32 * 256); };
    auto v_block_off = [&](int u) { return (uint32_t)((u >> 1) % 3) * kTileBytes + (uint32_t)(u & 1) * (2 * 4096); };

    bf16x8 kf[NKK], vf[2][NDB];
    auto load_kf = [&](int u) {
        const uint8_t *kb = Ks + k_block_off(u);
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) kf[kk] = *(const bf16x8 *)(kb + kaddr[kk]);
    };
    auto load_vf = [&](int u) {
        const uint8_t *vb = Vs + v_block_off(u);
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int db = 0; db < NDB; ++db)
                vf[st][db] = lds_read_tr8(vb + 4096 * st + vaddr[db][0], vb + 4096 * st + vaddr[db][1]);
    };

    f32x16 oacc[2][NDB];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int db = 0; db < NDB; ++db) oacc[r][db] = zero16;
    float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
    const float c2 = p.scale_log2;

    auto qk = [&](int r, f32x16 &s) {
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[r][kk], kk == 0 ? zero16 : s, 0, 0, 0);
    };
    auto pv = [&](int r, const bf16x8 (&pb)[2]) {
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int db = 0; db < NDB; ++db)
                oacc[r][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[st][db], pb[st], oacc[r][db], 0, 0, 0);
    };
    auto row_max = [&](const f32x16 &s) {
        float tmax = max3(s[0], s[1], s[2]);
#pragma unroll
        for (int e = 3; e < 15; e += 2) tmax = max3(tmax, s[e], s[e + 1]);
        tmax = fmaxf(tmax, s[15]);
        return fmaxf(tmax, xchg_half(tmax));
    };
    // raise the running max of group r to cover `cand`; rescale O and the row sum when it moved
    auto raise_max = [&](int r, float cand) {
        const float m_new = fmaxf(m_run[r], cand);
        if (__any(m_new > m_run[r])) {
            const float alpha = (m_run[r] == -INFINITY) ? 0.f : fast_exp2((m_run[r] - m_new) * c2);
            l_run[r] *= alpha;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[r][db][e] *= alpha;
            m_run[r] = m_new;
        }
    };
    // exponentials of one block against the running max; bf16 B operands of the two PV k-steps
    auto exps = [&](int r, f32x16 &s, bf16x8 (&pb)[2]) {
        const float mc = (m_run[r] == -INFINITY) ? 0.f : m_run[r] * c2;
        float psum = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            s[e] = fast_exp2(fmaf(s[e], c2, -mc));
            psum += s[e];
        }
        l_run[r] += psum;
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            f32x8 pf;
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[e] = s[8 * st + e];
            pb[st] = __builtin_convertvector(pf, bf16x8);
        }
    };
    auto tile_end = [&]() {
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    };

    // ---- prologue: tiles 0 and 1
    issue_tile(0);
    issue_tile(1);
    tile_end();

    // Leading blocks that no query of the workgroup has to mask: 32 u + 31 <= m0 + delta.
    // They are processed in whole tiles by the pipelined loop; the rest by the generic loop.
    const int first_lim = m0 + delta;
    const int t_hot = min((first_lim + 1) / kBN, n_tiles);
    int t = 0;

    if (t_hot > 0) {
        f32x16 sa, sb;
        bf16x8 pa[2], pb_[2];
        // fill: scores of block 0 for both groups, softmax of group a, fragments for the first phases
        load_kf(0);
        qk(0, sa);
        qk(1, sb);
        raise_max(0, row_max(sa));
        exps(0, sa, pa);
        float mcand_b = row_max(sb), mcand_a = -INFINITY;
        load_vf(0);
        if (n_tiles * 2 > 1) load_kf(1);

        for (; t < t_hot; ++t) {
            issue_tile(t + 2);
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
                const int u = 2 * t + blk;
                const bool last = (t == t_hot - 1) && (blk == 1);   // drain: nothing beyond block u
                if (!last) {
                    // phase A: matrix pipe on group a (scores of u+1, PV of u), vector ALU on group b
                    raise_max(1, mcand_b);
                    qk(0, sa);
                    pv(0, pa);
                    exps(1, sb, pb_);
                    mcand_a = row_max(sa);
                    // phase B: matrix pipe on group b, vector ALU on group a; fragments for the next block
                    raise_max(0, mcand_a);
                    qk(1, sb);
                    if (u + 2 < 2 * n_tiles) load_kf(u + 2);
                    pv(1, pb_);
                    load_vf(u + 1);
                    exps(0, sa, pa);
                    mcand_b = row_max(sb);
                } else {
                    raise_max(1, mcand_b);
                    pv(0, pa);
                    exps(1, sb, pb_);
                    pv(1, pb_);
                }
            }
            tile_end();
        }
    }

    // ---- remaining tiles (the diagonal region): per-group activity and masking, not pipelined
    for (; t < n_tiles; ++t) {
        issue_tile(t + 2);
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            const int u = 2 * t + blk;
            const int j0 = 32 * u;
            if (j0 <= grp_lim_max[1]) {          // group b sees at least as far as group a
                load_kf(u);
                load_vf(u);
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    if (j0 <= grp_lim_max[r]) {
                        f32x16 s;
                        bf16x8 pq[2];
                        qk(r, s);
                        if (j0 + 31 > grp_lim_min[r]) {
#pragma unroll
                            for (int e = 0; e < 16; ++e) {
                                const int j = j0 + 8 * (e >> 2) + 4 * hh + (e & 3);
                                if (j > lim[r]) s[e] = -INFINITY;
                            }
                        }
                        raise_max(r, row_max(s));
                        exps(r, s, pq);
                        pv(r, pq);
                    }
                }
            }
        }
        tile_end();
    }

    // ---- epilogue: normalise, write O (bf16) and LSE (fp32, natural log)
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const float l_tot = l_run[r] + xchg_half(l_run[r]);
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        if (qrow[r] < nq) {
            uint16_t *op = p.o + (int64_t)(qs + qrow[r]) * p.o_st + (int64_t)h * p.o_sh;
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
#pragma unroll
                for (int bq = 0; bq < 4; ++bq) {
                    f32x4 x;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = oacc[r][db][4 * bq + e] * inv;
                    const bf16x4 y = __builtin_convertvector(x, bf16x4);
                    *(bf16x4 *)(op + 32 * db + 8 * bq + 4 * hh) = y;
                }
            }
            if (hh == 0) {
                const float lse = l_tot > 0.f
                    ? (m_run[r] * c2 + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f
                    : -INFINITY;
                p.lse[(int64_t)h * p.total_q + qs + qrow[r]] = lse;
            }
        }
    }
#else
    (void)p;
#endif
}

}  // namespace pdd
