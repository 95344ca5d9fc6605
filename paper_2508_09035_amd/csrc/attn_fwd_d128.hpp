// Causal / GQA / ragged prefill attention, head_dim 128, tuned for gfx950.
//
// Same mathematics and the same register layout as the generic kernel in
// attn_fwd.hpp (S^T = K Q^T, lane = query, O^T = V^T P^T); what differs is the
// data movement and the instruction schedule:
//   * K and V tiles (64 keys x 256 B) go from HBM/L2 straight into LDS with
//     buffer_load ... lds (no staging registers, no ds_write); rows past the
//     end of the sequence read as zero through the buffer bounds check.
//   * Both tiles are row-major in LDS with a 16-byte-chunk XOR swizzle
//       chunk' = chunk ^ (((row & 3) << 2) | ((row >> 2) & 3))
//     which makes the K fragment reads (ds_read_b128, 16 rows per quarter
//     wave) and the V^T fragment reads (ds_read_b64_tr_b16, 4 rows x 64 B per
//     16 lanes) bank-conflict free without padding.
//   * V is transposed on the fly by the LDS transpose read, so V needs no
//     register shuffle.
//   * The loop is software pipelined: the QK^T MFMAs of tile j+1 are issued
//     together with the softmax VALU work of tile j, then the PV MFMAs of
//     tile j follow.
#pragma once
#include "attn_fwd.hpp"

namespace pdd {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

constexpr int kTileBytes = kBN * 256;   // one K or V tile in LDS
constexpr int kAttn128Smem = 4 * kTileBytes;

__device__ __forceinline__ int swz16(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

typedef __attribute__((address_space(3))) void *lds_ptr_t;

__device__ __forceinline__ bf16x8 lds_read_tr8(const uint8_t *lo, const uint8_t *hi)
{
    // two transposing 64-bit reads -> 8 bf16 (k-slots 0..3 from lo, 4..7 from hi)
    const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)lo);
    const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)hi);
    const s16x8 c = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, c);
}

template <int NWAVES>
__global__ __launch_bounds__(NWAVES * 64) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_fwd_d128_kernel(const AttnParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the body uses gfx950-only types; the host pass needs the stub only
    constexpr int D = 128;
    constexpr int BM = NWAVES * 32;
    constexpr int NKK = D / 16, NDB = D / 32;
    constexpr int NLD = 16 / NWAVES;     // buffer_load..lds instructions per tile per wave

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem128[];
    uint8_t *Ks = smem128;                    // [2][kTileBytes]
    uint8_t *Vs = smem128 + 2 * kTileBytes;   // [2][kTileBytes]

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
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, hh = lane >> 5;

    const int wave_q0 = m0 + 32 * wave;
    const int qrow = wave_q0 + n;
    const int qrow_c = min(qrow, nq - 1);
    const int lim = qrow_c + delta;
    const int wave_lim_max = min(wave_q0 + 31, nq - 1) + delta;
    const int wave_lim_min = min(wave_q0, nq - 1) + delta;
    const int kend = min(nk, min(m0 + BM, nq) + delta);
    const int n_tiles = kend > 0 ? (kend + kBN - 1) / kBN : 0;

    // ---- Q fragments (B operand)
    bf16x8 qf[NKK];
    {
        const uint16_t *qp = p.q + (int64_t)(qs + qrow_c) * p.q_st + (int64_t)h * p.q_sh + 8 * hh;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) qf[kk] = *(const bf16x8 *)(qp + 16 * kk);
    }

    // ---- buffer resources over this sequence's K / V rows of KV head g
    const uint16_t *kbase = p.k + (int64_t)ks * p.k_st + (int64_t)g * p.k_sh;
    const uint16_t *vbase = p.v + (int64_t)ks * p.v_st + (int64_t)g * p.v_sh;
    const uint32_t k_row_bytes = (uint32_t)p.k_st * 2u, v_row_bytes = (uint32_t)p.v_st * 2u;
    const uint32_t k_span = nk > 0 ? (uint32_t)(nk - 1) * k_row_bytes + 256u : 0u;
    const uint32_t v_span = nk > 0 ? (uint32_t)(nk - 1) * v_row_bytes + 256u : 0u;
    const __amdgpu_buffer_rsrc_t rsK = __builtin_amdgcn_make_buffer_rsrc((void *)kbase, 0, (int)k_span, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsV = __builtin_amdgcn_make_buffer_rsrc((void *)vbase, 0, (int)v_span, 0x00020000);

    // DMA lane mapping: instruction ci of wave w fills LDS rows 4q..4q+3, q = w + NWAVES*ci;
    // lane -> row 4q + lane/16, chunk position lane%16, which holds chunk pos ^ swz(row).
    uint32_t kvoff[NLD], vvoff[NLD];
#pragma unroll
    for (int ci = 0; ci < NLD; ++ci) {
        const int r = 4 * (wave + NWAVES * ci) + (lane >> 4);
        const int c = (lane & 15) ^ swz16(r);
        kvoff[ci] = (uint32_t)r * k_row_bytes + (uint32_t)c * 16u;
        vvoff[ci] = (uint32_t)r * v_row_bytes + (uint32_t)c * 16u;
    }
    auto issue_k = [&](int tile) {
        uint8_t *dst = Ks + (tile & 1) * kTileBytes;
        // the tile offset goes into the per-lane offset: only that one is range checked
        const uint32_t so = (uint32_t)tile * kBN * k_row_bytes;
#pragma unroll
        for (int ci = 0; ci < NLD; ++ci)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsK, (lds_ptr_t)(dst + 1024 * (wave + NWAVES * ci)), 16,
                                                     kvoff[ci] + so, 0, 0, 0);
    };
    auto issue_v = [&](int tile) {
        uint8_t *dst = Vs + (tile & 1) * kTileBytes;
        const uint32_t so = (uint32_t)tile * kBN * v_row_bytes;
#pragma unroll
        for (int ci = 0; ci < NLD; ++ci)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsV, (lds_ptr_t)(dst + 1024 * (wave + NWAVES * ci)), 16,
                                                     vvoff[ci] + so, 0, 0, 0);
    };

    // ---- LDS read addresses (bytes inside a tile)
    // K fragment (A operand of S^T): row n (+32 for the second block), chunk (2kk+hh) ^ swz(n)
    uint32_t kaddr[NKK];
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) kaddr[kk] = (uint32_t)n * 256u + (uint32_t)(((2 * kk + hh) ^ swz16(n)) * 16);
    // V^T fragment (A operand of O^T) through the transposing read: the 16 lanes of group
    // gamma = lane/16 address 4 keys x 16 dims; source lane s reads key (s>>2), dims 4(s&3)..+3.
    // Keys of step st, half hh, read eg: 16 st + 8 eg + 4 hh + (s>>2).
    uint32_t vaddr[NDB][2];
    {
        const int s16 = lane & 15, dhalf = (lane >> 4) & 1;
#pragma unroll
        for (int eg = 0; eg < 2; ++eg) {
            const int row = 8 * eg + 4 * hh + (s16 >> 2);          // + 16 st
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                const int chunk = 4 * db + 2 * dhalf + ((s16 & 3) >> 1);
                vaddr[db][eg] = (uint32_t)row * 256u + (uint32_t)((chunk ^ swz16(row)) * 16) + 8u * (s16 & 1);
            }
        }
    }

    f32x16 oacc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[db][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float c2 = p.scale_log2;

    auto qk_tile = [&](int tile, f32x16 &s0, f32x16 &s1) {
        const uint8_t *kb = Ks + (tile & 1) * kTileBytes;
        const bool blk1 = tile * kBN + 32 <= wave_lim_max;
#pragma unroll
        for (int e = 0; e < 16; ++e) { s0[e] = 0.f; s1[e] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
            const bf16x8 a = *(const bf16x8 *)(kb + kaddr[kk]);
            s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s0, 0, 0, 0);
        }
        if (blk1) {
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk) {
                const bf16x8 a = *(const bf16x8 *)(kb + 32 * 256 + kaddr[kk]);
                s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s1, 0, 0, 0);
            }
        }
    };

    if (n_tiles > 0) {
        issue_k(0);
        issue_v(0);
        if (n_tiles > 1) issue_k(1);
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    f32x16 s0, s1;
    if (n_tiles > 0) qk_tile(0, s0, s1);   // tile 0 is visible to every wave

    for (int it = 0; it < n_tiles; ++it) {
        const int j0 = it * kBN;
        const bool cur_active = j0 <= wave_lim_max;
        const bool nxt_active = it + 1 < n_tiles && j0 + kBN <= wave_lim_max;
        // the buffers these tiles land in were last read one iteration ago
        if (it + 1 < n_tiles) issue_v(it + 1);
        if (it + 2 < n_tiles) issue_k(it + 2);

        f32x16 t0 = s0, t1 = s1;
        if (nxt_active) qk_tile(it + 1, t0, t1);

        if (cur_active) {
            const bool blk1 = (j0 + 32 <= wave_lim_max);
            if (j0 + kBN - 1 > wave_lim_min) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int j = j0 + 8 * (e >> 2) + 4 * hh + (e & 3);
                    if (j > lim) s0[e] = -INFINITY;
                    if (j + 32 > lim) s1[e] = -INFINITY;
                }
            }
            float tmax = max3(s0[0], s0[1], s0[2]);
#pragma unroll
            for (int e = 3; e < 15; e += 2) tmax = max3(tmax, s0[e], s0[e + 1]);
#pragma unroll
            for (int e = 0; e < 16; e += 2) tmax = max3(tmax, s1[e], s1[e + 1]);
            tmax = fmaxf(tmax, s0[15]);
            tmax = fmaxf(tmax, xchg_half(tmax));
            const float m_new = fmaxf(m_run, tmax);
            if (__any(m_new > m_run)) {
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

            const uint8_t *vb = Vs + (it & 1) * kTileBytes;
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                if (st >= 2 && !blk1) break;
                f32x8 pf;
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[e] = (st < 2) ? s0[8 * (st & 1) + e] : s1[8 * (st & 1) + e];
                const bf16x8 pb = __builtin_convertvector(pf, bf16x8);
#pragma unroll
                for (int db = 0; db < NDB; ++db) {
                    const bf16x8 a = lds_read_tr8(vb + 4096 * st + vaddr[db][0], vb + 4096 * st + vaddr[db][1]);
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, oacc[db], 0, 0, 0);
                }
            }
        }
        s0 = t0;
        s1 = t1;
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    }

    // ---- epilogue
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
#else
    (void)p;
#endif
}

}  // namespace pdd
