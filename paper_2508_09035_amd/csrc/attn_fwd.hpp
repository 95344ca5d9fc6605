// Causal / GQA / ragged prefill attention for gfx950 (flash-style forward), head_dim 64 or 128.
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
//   (sequence, query head); a sequence's query tiles are aligned to its end, so
//   that rows a ragged length leaves empty fall into the tile with the fewest
//   keys; key/value tiles of 64 keys stream through LDS.
//   Per 32-key block a wave computes S^T = K Q^T with v_mfma_f32_32x32x16_bf16
//   (A = K rows from LDS, B = Q fragments held in registers), so lane l owns
//   query (l % 32) and the 16 accumulator registers hold 16 different keys:
//   row max / row sum are in-lane reductions plus one exchange between lanes
//   l and l+32.  O^T = V^T P^T reuses those registers directly as the B
//   operand (the contraction index "key" may be permuted freely as long as the
//   V^T fragments are read with the same permutation).
//
// Data movement and instruction schedule
//   * K and V tiles (64 keys x 2 D bytes) go from HBM/L2 straight into LDS with
//     buffer_load ... lds (no staging registers, no ds_write); rows past the
//     end of the sequence read as zero through the buffer bounds check.  The
//     workgroup's Q rows take the same way once, in the layout of K tiles, and
//     O leaves through LDS as whole rows: every global access of the kernel
//     moves whole rows, 16 bytes per lane.
//   * Both tiles are row-major in LDS with a 16-byte-chunk XOR swizzle,
//       D = 128 (16 chunks per row):  chunk' = chunk ^ (((row & 3) << 2) | ((row >> 2) & 3))
//       D = 64  (8 chunks per row):   chunk' = chunk ^ ((((row >> 1) & 1) << 2) | ((row >> 2) & 3))
//     which makes the K fragment reads (ds_read_b128, 16 rows per quarter
//     wave) and the V^T fragment reads (ds_read_b64_tr_b16, 4 rows x 64 B per
//     32 lanes) bank-conflict free without padding.
//   * V is transposed on the fly by the LDS transpose read, so V needs no
//     register shuffle.
//   * The loop is software pipelined: the QK^T MFMAs of block j+1 are issued
//     together with the softmax VALU work of block j, then the PV MFMAs of
//     block j follow.  The tiles at the diagonal run through the same pipeline
//     with the causal mask applied to the blocks computed ahead.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

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

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

constexpr int kAttnBufs = 3;             // K and V tiles are triple buffered
constexpr int kSweepBufs = 6;            // importance sweep: K tiles rotate through six buffers,
constexpr int kSweepAhead = 5;           //   tile t+5 is requested while tile t is summed
template <int D>
struct AttnSmem {
    static constexpr int TILE = kBN * D * 2;                       // one K or V tile in LDS, bytes
    static constexpr int BYTES = (2 * kAttnBufs + 1) * TILE;     // + the fourth Q slot of an 8-wave workgroup
    static constexpr int SWEEP_BYTES = (kSweepBufs + 1) * TILE;    // + exchange area
};
constexpr float kLazyLog2 = 8.0f;        // a row's softmax reference may lag its running max by a factor 2^8

// chunk swizzle of LDS row `row` (see the head of this file)
template <int D>
__device__ __forceinline__ int swz_row(int row)
{
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}

typedef __attribute__((ext_vector_type(4))) int32_t i32x4;

// Raw buffer descriptor (base, num_records in bytes, untyped dword access) held in SGPRs.
__device__ __forceinline__ i32x4 make_rsrc(const void *base, uint32_t bytes)
{
    const uint64_t a = (uint64_t)base;
    i32x4 r;
    r.x = __builtin_amdgcn_readfirstlane((int32_t)(uint32_t)a);
    r.y = __builtin_amdgcn_readfirstlane((int32_t)((uint32_t)(a >> 32) & 0xffffu));
    r.z = __builtin_amdgcn_readfirstlane((int32_t)bytes);
    r.w = 0x00020000;
    return r;
}

// 16 bytes per lane from the buffer straight into LDS at lds_addr + 16 * lane
// (lds_addr wave-uniform).  Out-of-range lanes write zeros.  Written as inline
// assembly so that the transfer stays asynchronous: completion is awaited with
// an explicit s_waitcnt vmcnt(0) before the workgroup barrier that publishes
// the tile.  M0 is declared clobbered, so the compiler neither keeps a value in it across
// the transfer nor misses the wait state after the write.
__device__ __forceinline__ void dma16_to_lds(i32x4 rsrc, uint32_t lds_addr, uint32_t voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc)
                 : "memory", "m0");
}

__device__ __forceinline__ uint32_t lds_addr_of(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const uint8_t *)p;
}

__device__ __forceinline__ bf16x8 lds_read_tr8(uint32_t lo, uint32_t hi)
{
    // two transposing 64-bit reads -> 8 bf16 (k-slots 0..3 from lo, 4..7 from hi); lo / hi are
    // LDS byte addresses, so that constant parts fold into the instruction's offset field
    const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(uintptr_t)lo);
    const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(uintptr_t)hi);
    const s16x8 c = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, c);
}

template <int D, int NWAVES, bool IMP = false>
__global__ __launch_bounds__(NWAVES * 64) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_fwd_kernel(const AttnParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the body uses gfx950-only types; the host pass needs the stub only
    static_assert(D == 64 || D == 128, "head_dim 64 or 128");
    constexpr int ROWB = 2 * D;                 // bytes of one K or V row
    constexpr int CH = D / 8;                   // 16-byte chunks per row
    constexpr int RPI = 1024 / ROWB;            // rows one buffer_load ... lds instruction fills
    constexpr int kTileBytes = AttnSmem<D>::TILE;
    constexpr int BM = NWAVES * 32;
    constexpr int NKK = D / 16, NDB = D / 32;
    constexpr int NLD = kBN / RPI / NWAVES;     // buffer_load..lds instructions per tile per wave

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem_attn[];
    uint8_t *Ks = smem_attn;                               // [3][kTileBytes], tile t in buffer t % 3
    uint8_t *Vs = smem_attn + kAttnBufs * kTileBytes;   // [3][kTileBytes]

    // Workgroups go to the 8 XCDs round robin, each XCD with an L2 of its own.  KV head fastest:
    // where the number of KV heads divides 8 or is a multiple of 8, all workgroups that share the
    // K and V of a KV head run on the same XCD(s) and find its tiles in that L2; then the query
    // heads of the group, the sequence, and the query tiles from the last (longest) down.
    int bid = blockIdx.x;
    const int g = bid % p.Hkv;  bid /= p.Hkv;
    const int hg = bid % p.G;   bid /= p.G;
    const int b = bid % p.B;    bid /= p.B;
    const int t = p.n_qtiles - 1 - bid;
    const int h = g * p.G + hg;

    const int qs = min(p.cu_q[b], p.total_q), qe = min(p.cu_q[b + 1], p.total_q);
    const int ks = min(p.cu_k[b], p.total_k), ke = min(p.cu_k[b + 1], p.total_k);
    const int nq = qe - qs, nk = ke - ks;
    // The sequence's query tiles are aligned to its END: tile t of n_qt holds rows m0 .. m0 + BM - 1
    // with m0 = nq - (n_qt - t) BM, and where nq is not a multiple of BM the rows below 0, which
    // do not exist, fall into tile 0, the workgroup with the fewest keys (aligned to the start,
    // the empty rows would sit in the last tile and ride along through all of its key tiles).
    const int n_qt = (nq + BM - 1) / BM;
    const int m0 = nq - (n_qt - t) * BM;
    const int tid = threadIdx.x;
    // importance sweep: this workgroup's slice of the partial column sums, at its sequence
    float *const part_row = IMP
        ? p.imp_part + ((int64_t)(hg * p.n_qtiles + t) * p.Hkv + g) * p.total_k + ks : nullptr;
    if (t >= n_qt || nq <= 0) {
        if constexpr (IMP)   // no query rows here: the slice still has to read as zero
            for (int j = tid; j < nk; j += NWAVES * 64) part_row[j] = 0.f;
        return;
    }
    const int delta = nk - nq;

    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, hh = lane >> 5;

    const int wave_q0 = m0 + 32 * wave;
    const int qrow = wave_q0 + n;
    const int qrow_c = max(qrow, 0);               // a row that does not exist computes like row 0; nothing of it is stored
    const int lim = qrow_c + delta;
    const int wave_lim_max = max(wave_q0 + 31, 0) + delta;
    const int wave_lim_min = max(wave_q0, 0) + delta;
    const int kend = min(nk, m0 + BM + delta);
    const int n_tiles = kend > 0 ? (kend + kBN - 1) / kBN : 0;

    // ---- buffer resources over this sequence's K / V rows of KV head g
    const uint16_t *kbase = p.k + (int64_t)ks * p.k_st + (int64_t)g * p.k_sh;
    const uint16_t *vbase = p.v + (int64_t)ks * p.v_st + (int64_t)g * p.v_sh;
    const uint32_t k_row_bytes = (uint32_t)p.k_st * 2u, v_row_bytes = (uint32_t)p.v_st * 2u;
    const uint32_t k_span = nk > 0 ? (uint32_t)(nk - 1) * k_row_bytes + (uint32_t)ROWB : 0u;
    const uint32_t v_span = nk > 0 ? (uint32_t)(nk - 1) * v_row_bytes + (uint32_t)ROWB : 0u;
    const uint32_t ks_lds = lds_addr_of(Ks), vs_lds = lds_addr_of(Vs);

    // DMA lane mapping: instruction ci of wave w fills the RPI LDS rows RPI q .. RPI q + RPI - 1,
    // q = w + NWAVES*ci; lane -> row RPI q + lane / CH, chunk position lane % CH, which holds
    // chunk pos ^ swz(row).
    uint32_t kvoff[NLD], vvoff[NLD];
#pragma unroll
    for (int ci = 0; ci < NLD; ++ci) {
        const int r = RPI * (wave + NWAVES * ci) + lane / CH;
        const int c = (lane % CH) ^ swz_row<D>(r);
        kvoff[ci] = (uint32_t)r * k_row_bytes + (uint32_t)c * 16u;
        vvoff[ci] = (uint32_t)r * v_row_bytes + (uint32_t)c * 16u;
    }
    // The tile's offset goes into the descriptor (scalar arithmetic): base advanced by the tile,
    // num_records reduced by the same amount, so that the range check still ends at the sequence's
    // last row and the per-lane offsets stay constant.
    auto tile_rsrc = [&](const uint16_t *base, uint32_t span, uint32_t so) {
        // span - min(so, span) on the scalar unit (the compiler turns the C form into a saturating
        // subtract, which exists only on the vector unit and then needs a readfirstlane)
        uint32_t left;
        asm("s_min_u32 %0, %1, %2\n\ts_sub_u32 %0, %2, %0" : "=&s"(left) : "s"(so), "s"(span) : "scc");
        return make_rsrc((const uint8_t *)base + so, left);
    };
    auto issue_k = [&](int tile, int buf) {
        const i32x4 rs = tile_rsrc(kbase, k_span, (uint32_t)tile * kBN * k_row_bytes);
#pragma unroll
        for (int ci = 0; ci < NLD; ++ci)
            dma16_to_lds(rs, ks_lds + buf * kTileBytes + 1024 * (wave + NWAVES * ci), kvoff[ci]);
    };
    auto issue_v = [&](int tile, int buf) {
        const i32x4 rs = tile_rsrc(vbase, v_span, (uint32_t)tile * kBN * v_row_bytes);
#pragma unroll
        for (int ci = 0; ci < NLD; ++ci)
            dma16_to_lds(rs, vs_lds + buf * kTileBytes + 1024 * (wave + NWAVES * ci), vvoff[ci]);
    };

    // ---- LDS read addresses (bytes inside a tile)
    // K fragment (A operand of S^T): row n (+32 for the second block), chunk (2kk+hh) ^ swz(n)
    uint32_t kaddr[NKK];
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) kaddr[kk] = (uint32_t)(n * ROWB + ((2 * kk + hh) ^ swz_row<D>(n)) * 16);
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
                vaddr[db][eg] = vs_lds + (uint32_t)(row * ROWB + (chunk ^ swz_row<D>(row)) * 16) + 8u * (s16 & 1);
                // kept as one value each: left to itself the compiler splits an address into a part
                // per read group and a part per dim block and adds the two again before every read
                asm volatile("" : "+v"(vaddr[db][eg]));
            }
        }
    }

    // ---- Q fragments (B operand).  The wave's 32 rows come in whole rows, RPI per instruction,
    // through LDS in the layout of half a K tile (read per lane from global memory, a row per
    // lane, every load instruction touches 32 rows 32 bytes at a time and the loads of a
    // workgroup take longer than the first K and V tiles).  They land in buffers that the first
    // K and V requests below leave alone; rows below 0 read row 0 (a wave without rows: zeros).
    // tile-sized LDS slots 2, 4, 5, 6 (K buffer 2, V buffers 1 and 2, one behind them), two waves each
    const uint32_t q_lds_off = (uint32_t)((wave < 2 ? 2 : 3 + (wave >> 1)) * kTileBytes + (wave & 1) * 32 * ROWB);
    bf16x8 qf[NKK];
    auto issue_q = [&]() {
        const int q_first = max(wave_q0, 0);        // the wave's first existing row
        const uint16_t *qbase = p.q + (int64_t)(qs + q_first) * p.q_st + (int64_t)h * p.q_sh;
        const uint32_t q_row_bytes = (uint32_t)p.q_st * 2u;
        const int q_rows = wave_q0 + 32 - q_first;
        const uint32_t q_span = q_rows > 0 ? (uint32_t)(q_rows - 1) * q_row_bytes + (uint32_t)ROWB : 0u;
        const i32x4 rs = make_rsrc(qbase, q_span);
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) {
            const int r = RPI * i + lane / CH;
            const int c = (lane % CH) ^ swz_row<D>(r);
            const int r_rel = max(wave_q0 + r - q_first, 0);
            dma16_to_lds(rs, ks_lds + q_lds_off + 1024 * i, (uint32_t)r_rel * q_row_bytes + (uint32_t)c * 16u);
        }
    };

    f32x16 oacc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[db][e] = 0.f;
    // Online-softmax state of this lane's query, kept in the log2 domain: every score enters as
    //   t = s * c2 + ref      (c2 = softmax scale * log2 e, ref = minus the row's reference exponent)
    // and contributes 2^t.  The reference only has to keep 2^t in range, it need not be the
    // running max: it is set by the first block that holds a visible key and renewed when a
    // block's largest t exceeds kLazyLog2 (probabilities relative to it stay below 2^kLazyLog2,
    // far inside the range of fp32 sums and bf16 operands), so O and the row sums are rescaled a
    // few times per row instead of whenever a max moves.
    float l_part[4] = {0.f, 0.f, 0.f, 0.f};   // four interleaved partial row sums (short add chains)
    const float c2 = p.scale_log2;
    float ref = 0.f;                           // 0 until the row has a reference
    float thr = -INFINITY;                     // a block max above it renews the reference: -inf, then kLazyLog2
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // S^T of the 32-key block at byte offset `koff` of the K buffers
    auto qk_block = [&](uint32_t koff, f32x16 &s) {
        const uint8_t *kb = Ks + koff;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
            const bf16x8 a = *(const bf16x8 *)(kb + kaddr[kk]);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], kk == 0 ? zero16 : s, 0, 0, 0);
        }
    };

    // t = s * c2 + ref in place
    auto to_log2 = [&](f32x16 &s) {
#pragma unroll
        for (int e = 0; e < 16; ++e) s[e] = fmaf(s[e], c2, ref);
    };

    // largest entry of the query's row in this block; its keys are spread over this lane and
    // lane ^ 32.  Short dependency chains: a 3-level tree of v_max3 instead of one serial chain.
    auto row_max = [&](const f32x16 &s) {
        const float t0 = max3(s[0], s[1], s[2]), t1 = max3(s[4], s[5], s[6]);
        const float t2 = max3(s[8], s[9], s[10]), t3 = max3(s[12], s[13], s[14]);
        const float u0 = max3(t0, t1, s[3]), u1 = max3(t2, t3, s[7]);
        const float tmax = max3(max3(u0, u1, s[11]), s[15], s[15]);
        const uint32_t u = __float_as_uint(tmax);
        const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
        return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    };

    // Rare and wave-uniform: the rows whose block max t_max exceeds their threshold take it as
    // their new reference; O, the row sums and the block `blk` (already in the log2 domain) move
    // with it.  Rows without a reference (thr = -inf, nothing accumulated yet) get their first
    // one the same way; a block in which a row sees no key (t_max = -inf) changes nothing.
    auto renew = [&](float t_max, f32x16 &blk) {
        const bool up = t_max > thr;
        const float shift = up ? t_max : 0.f;
        const float alpha = fast_exp2(-shift);
#pragma unroll
        for (int i = 0; i < 4; ++i) l_part[i] *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[db][e] *= alpha;
#pragma unroll
        for (int e = 0; e < 16; ++e) blk[e] -= shift;
        ref -= shift;
        thr = up ? kLazyLog2 : thr;
    };

    // A wave all of whose rows lie below 0 (a chunk or a first tile shorter than the workgroup)
    // has nothing to compute or store: it only makes its share of the K and V requests and meets
    // the others at their barriers, two before the first tile and one per tile, and leaves the
    // matrix pipe to the waves with rows.  (With the importance sweep the wave stays on the
    // common path: the sweep needs it as one of the waves that add up a tile's column sums.)
    if constexpr (!IMP) {
        if (wave_q0 + 31 < 0) {
            if (n_tiles > 0) issue_k(0, 0);
            if (n_tiles > 0) issue_v(0, 0);
            if (n_tiles > 1) issue_k(1, 1);
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            __syncthreads();
            for (int it = 0; it < n_tiles; ++it) {
                if (it + 1 < n_tiles) issue_v(it + 1, (it + 1) % 3);
                if (it + 2 < n_tiles) issue_k(it + 2, (it + 2) % 3);
                __builtin_amdgcn_s_waitcnt(0);
                __syncthreads();
            }
            return;
        }
    }

    // Requests in the order of their first use.  The first barrier waits for K tile 0 and the Q
    // rows only (loads return in order: the younger requests may still be open); the first QK
    // block runs while V tile 0 and K tile 1 arrive, and the second barrier publishes those.
    if (n_tiles > 0) issue_k(0, 0);
    issue_q();
    if (n_tiles > 1) {
        issue_v(0, 0);
        issue_k(1, 1);
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(2 * NLD) : "memory");
    } else {
        if (n_tiles > 0) issue_v(0, 0);
        __builtin_amdgcn_s_waitcnt(0);
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) qf[kk] = *(const bf16x8 *)(smem_attn + q_lds_off + kaddr[kk]);

    // Scores are pipelined per 32-key block u = 2*tile + blk: while block u goes
    // through softmax and PV, the MFMAs of block u+1 are already issued.  Tile t
    // lives in LDS buffer t % 3; at every tile boundary the current block is in sA.
    f32x16 sA = zero16, sB = zero16;
    if (n_tiles > 0) qk_block(0, sA);   // every wave has rows that see block 0
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();                    // V tile 0, K tile 1; the next requests overwrite the Q rows

    // ---- hot tiles: those that no wave of the workgroup has to mask (fully visible to the
    // workgroup's first existing query: 64 (t+1) - 1 <= max(m0, 0) + delta) and that have a
    // successor tile.
    const int first_lim = max(m0, 0) + delta;
    const int n_hot = max(0, min((first_lim + 1) / kBN, n_tiles - 1));   // tiles 0 .. n_hot-1

    // The block `cur` arrives in the log2 domain (see above): the scale-and-shift and the row max
    // of a block are done one phase before its exponentials, while the previous PV MFMAs run, so
    // that the exponentials never wait for a max.  LDS fragment reads are issued a phase ahead of
    // the MFMAs that consume them: the V^T fragments of `cur` before the QK MFMAs of `nxt`, the K
    // fragments of the block after `nxt` (`kf`) before the PV MFMAs of `cur`.
    bf16x8 kf[NKK];
    auto load_kf = [&](uint32_t koff) {
        const uint8_t *kb = Ks + koff;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) kf[kk] = *(const bf16x8 *)(kb + kaddr[kk]);
    };
    // The wave runs at raised issue priority while it has the exponentials to do and at normal
    // priority during its PV MFMAs (measured: 1 % on the 32k prompt, 3 % on constant inputs).
    auto pipe_half = [&](auto mask_c, f32x16 &cur, f32x16 &nxt, uint32_t k_next2, uint32_t v_cur, const int l_nxt, const bool hidden) __attribute__((always_inline)) {
        constexpr bool MASK = decltype(mask_c)::value;
        __builtin_amdgcn_s_setprio(1);
        bf16x8 vf[2][NDB];
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int db = 0; db < NDB; ++db)
                vf[st][db] = lds_read_tr8(vaddr[db][0] + v_cur + 16 * ROWB * st, vaddr[db][1] + v_cur + 16 * ROWB * st);
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
            nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], kk == 0 ? zero16 : nxt, 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 16; ++e) cur[e] = fast_exp2(cur[e]);   // cur is in the log2 domain
        bf16x8 pb[2];
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            f32x8 pf;
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[e] = cur[8 * st + e];
            pb[st] = __builtin_convertvector(pf, bf16x8);
        }
        // Issue order of this phase, pinned: after every QK MFMA two exponentials, two V^T
        // fragment reads and one bf16 pack.  Left to itself the compiler bunches the exponentials
        // behind the first MFMAs and the reads behind the middle ones, and the two waves of a SIMD
        // then queue for the same unit (measured: 10 % fewer cycles on constant inputs, 2.5 % less
        // time on the 32k prompt, where the clock gives way as the matrix pipe fills).
#pragma unroll
        for (int i = 0; i < NKK; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);          // 1 MFMA
            __builtin_amdgcn_sched_group_barrier(0x400, 16 / NKK, 0);   // transcendental
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);          // 2 DS reads
            __builtin_amdgcn_sched_group_barrier(0x002, 8 / NKK, 0);    // VALU (bf16 packs)
        }
        __builtin_amdgcn_s_setprio(0);
        load_kf(k_next2);
        float t_max;
        if constexpr (!MASK) {
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const bf16x8 pbs = pb[st];
#pragma unroll
                for (int db = 0; db < NDB; ++db)
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[st][db], pbs, oacc[db], 0, 0, 0);
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) l_part[e & 3] += cur[e];      // row sums: also in this phase
            // The next block enters the log2 domain here, in the phase whose VALU is otherwise idle,
            // against the present reference (nothing here depends on the check below, so all of it
            // can be issued between the PV MFMAs).
            to_log2(nxt);
            t_max = row_max(nxt);
            // same for this phase: after every PV MFMA one K fragment read and five of the
            // additions, multiply-adds and max operations above
#pragma unroll
            for (int i = 0; i < 2 * NDB; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);              // 1 MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);              // 1 DS read
                __builtin_amdgcn_sched_group_barrier(0x002, 40 / (2 * NDB), 0); // VALU
            }
        } else {
            // The same work in two parts, with the mask between them for the waves that have a
            // hidden key in the block (a branch every lane of the wave takes alike): key
            // 8 (e / 4) + 4 hh + e % 4 of the block is hidden from the row iff it exceeds l_nxt + 4 hh.
            constexpr int NA = 2 * NDB - 2;       // PV MFMAs before the branch
#pragma unroll
            for (int i = 0; i < NA; ++i)
                oacc[i % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i / NDB][i % NDB], pb[i / NDB], oacc[i % NDB], 0, 0, 0);
#pragma unroll
            for (int e = 0; e < 16; ++e) l_part[e & 3] += cur[e];
            to_log2(nxt);
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                    // 1 MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, (NKK + NA - 1) / NA, 0);  // DS reads
                __builtin_amdgcn_sched_group_barrier(0x002, (32 + NA - 1) / NA, 0);   // VALU
            }
            // the row sums are complete here (left alone, their additions sink behind the branch and
            // pile up after the last two MFMAs)
            asm volatile("" : "+v"(l_part[0]), "+v"(l_part[1]), "+v"(l_part[2]), "+v"(l_part[3]));
            if (hidden) {
                asm volatile("" ::: "memory");     // stays a branch
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    nxt[e] = 8 * (e >> 2) + (e & 3) > l_nxt ? -INFINITY : nxt[e];
            }
#pragma unroll
            for (int i = NA; i < 2 * NDB; ++i)
                oacc[i % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i / NDB][i % NDB], pb[i / NDB], oacc[i % NDB], 0, 0, 0);
            t_max = row_max(nxt);
#pragma unroll
            for (int i = NA; i < 2 * NDB; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);              // 1 MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);              // VALU
            }
        }
        if (__any(t_max > thr)) renew(t_max, nxt);
    };
    auto hot_tile = [&](auto par_c, const int it) {
        constexpr int PAR = decltype(par_c)::value;
        constexpr int P1 = (PAR + 1) % 3, P2 = (PAR + 2) % 3;
        issue_v(it + 1, P1);
        if (it + 2 < n_tiles) issue_k(it + 2, P2);
        pipe_half(std::false_type{}, sA, sB, P1 * kTileBytes, PAR * kTileBytes, 0, false);
        pipe_half(std::false_type{}, sB, sA, P1 * kTileBytes + 32 * ROWB, PAR * kTileBytes + 32 * ROWB, 0, false);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    };
    // The same pipeline for the tiles at and next to the diagonal: the blocks computed ahead
    // are masked as they enter the log2 domain, before their row max is taken.  A block past the
    // row's last visible key, past the wave's last row or past the last tile (whose buffer holds
    // stale rows) comes out all -inf: it renews nothing and adds zeros.  A wave none of whose rows
    // sees the tile only takes part in the requests and the barrier.
    const int lim4 = lim - 4 * hh;
    auto masked_tile = [&](auto par_c, const int it) {
        constexpr int PAR = decltype(par_c)::value;
        constexpr int P1 = (PAR + 1) % 3, P2 = (PAR + 2) % 3;
        if (it + 1 < n_tiles) issue_v(it + 1, P1);
        if (it + 2 < n_tiles) issue_k(it + 2, P2);
        if (kBN * it <= wave_lim_max) {
            const int l1 = lim4 - (kBN * it + 32);
            const int w1 = wave_lim_min - (kBN * it + 32);      // the same for the wave's first row
            pipe_half(std::true_type{}, sA, sB, P1 * kTileBytes, PAR * kTileBytes, l1, w1 < 31);
            pipe_half(std::true_type{}, sB, sA, P1 * kTileBytes + 32 * ROWB, PAR * kTileBytes + 32 * ROWB, l1 - 32, w1 < 63);
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    };
    // The first block: masked where it touches the diagonal, then every row takes its first
    // reference from it (key 0 is visible to every row).
    int it = 0;
    if (n_tiles > 0) {
        if (31 > wave_lim_min) {
#pragma unroll
            for (int e = 0; e < 16; ++e)
                sA[e] = 8 * (e >> 2) + (e & 3) > lim4 ? -INFINITY : sA[e];
        }
        to_log2(sA);
        renew(row_max(sA), sA);
        load_kf(32 * ROWB);
    }
    // Plain tiles: the two blocks a tile computes ahead (its own second and the next tile's
    // first) are visible in full to every row of the workgroup, i.e. all hot tiles but the last.
    const int n_plain = max(0, n_hot - 1) / 3 * 3;   // whole rounds of the three LDS buffers
    for (; it < n_plain; it += 3) {
        hot_tile(std::integral_constant<int, 0>{}, it);
        hot_tile(std::integral_constant<int, 1>{}, it + 1);
        hot_tile(std::integral_constant<int, 2>{}, it + 2);
    }
    // ---- the last hot tiles and the diagonal region
    for (; it < n_tiles; it += 3) {
        masked_tile(std::integral_constant<int, 0>{}, it);
        if (it + 1 < n_tiles) masked_tile(std::integral_constant<int, 1>{}, it + 1);
        if (it + 2 < n_tiles) masked_tile(std::integral_constant<int, 2>{}, it + 2);
    }

    // ---- epilogue
    const float l_run = (l_part[0] + l_part[1]) + (l_part[2] + l_part[3]);
    const float l_tot = l_run + xchg_half(l_run);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    // O leaves through LDS (the K and V buffers are free now): each wave lays its 32 rows out row
    // by row in a slice of its own, 16-byte chunk c of row r at position c ^ (r mod CH), and then
    // stores RPI whole rows per instruction, 16 bytes per lane.  (Stored straight from the
    // accumulator layout, a row per lane, every store instruction touches 32 rows 16 bytes at a
    // time, and the compute unit spends the time of two to three key tiles issuing them.)
    {
        uint8_t *ost = smem_attn + wave * (32 * ROWB);
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
#pragma unroll
            for (int bq = 0; bq < 4; ++bq) {
                f32x4 x;
#pragma unroll
                for (int r = 0; r < 4; ++r) x[r] = oacc[db][4 * bq + r] * inv;
                const bf16x4 y = __builtin_convertvector(x, bf16x4);
                *(bf16x4 *)(ost + n * ROWB + (((4 * db + bq) ^ (n & (CH - 1))) * 16) + 8 * hh) = y;
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the slice is read by other lanes of the wave
        const int sr = lane / CH, sc = lane % CH;
        uint16_t *op = p.o + (int64_t)(qs + wave_q0 + sr) * p.o_st + (int64_t)h * p.o_sh + 8 * sc;
        u32x4 x[32 / RPI];
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i) {
            const int row = RPI * i + sr;
            x[i] = *(const u32x4 *)(ost + row * ROWB + ((sc ^ (row & (CH - 1))) * 16));
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // all reads before the first store
#pragma unroll
        for (int i = 0; i < 32 / RPI; ++i)
            if (wave_q0 + RPI * i + sr >= 0) *(u32x4 *)(op + (int64_t)(RPI * i) * p.o_st) = x[i];
    }
    if (qrow >= 0 && hh == 0) {
        const float lse = l_tot > 0.f
            ? (__builtin_amdgcn_logf(l_tot) - ref) * 0.6931471805599453f
            : -INFINITY;
        p.lse[(int64_t)h * p.total_q + qs + qrow] = lse;
    }
    if constexpr (IMP) {   // the second sweep's first requests overwrite the slices
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __syncthreads();
    }

    // ---- importance sweep (paper Section 3.2, token importance of an observation window that
    // covers every query of the call): with the final log-sum-exp of its 32 rows in hand, each
    // wave walks the same K tiles again, recomputes S = Q K^T with the operands exchanged (lane =
    // key, registers = the wave's 32 query rows), turns it into the normalised probabilities and
    // adds them up along the query dimension.  The waves' column sums of a 64-key tile meet
    // in LDS; one wave adds them in the fixed order wave 0, 1, ... and writes the tile's 64 sums.
    // No atomics: the result does not depend on timing.
    if constexpr (IMP) {
        // LDS: K tiles now rotate through kSweepBufs buffers (the K and V buffers of the first
        // sweep, contiguous); the log-sum-exp exchange and the column sums lie behind them.  A step
        // is short (D / 8 MFMAs per wave), so a tile is requested five steps before its first use and
        // the wait at the end of a step leaves the two youngest requests in flight.
        float *lse_sh = (float *)(smem_attn + kSweepBufs * kTileBytes);          // [NWAVES][32]
        float *red = (float *)(smem_attn + kSweepBufs * kTileBytes + 1024);      // [2][64][NWAVES]
        // a row's probabilities are 2^(s * c2 - lse2); rows past the end or without a visible key give 0
        const float lse2 = (qrow >= 0 && l_tot > 0.f) ? __builtin_amdgcn_logf(l_tot) - ref : INFINITY;
        if (hh == 0) lse_sh[wave * 32 + n] = lse2;
        for (int tl = 0; tl < kSweepAhead; ++tl) issue_k(tl, tl);   // tiles past the end read as zero
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        float nl[16];                              // minus lse2 of the rows this lane's registers hold
#pragma unroll
        for (int bq = 0; bq < 4; ++bq) {
            const f32x4 x = *(const f32x4 *)(lse_sh + wave * 32 + 8 * bq + 4 * hh);
#pragma unroll
            for (int r = 0; r < 4; ++r) nl[4 * bq + r] = -x[r];
        }
        // S of the 32-key block at byte offset `koff`: rows 8 (e / 4) + 4 hh + e % 4 of the wave, key n
        auto qk_rows = [&](uint32_t koff, f32x16 &s) {
            const uint8_t *kb = Ks + koff;
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk) {
                const bf16x8 kfrag = *(const bf16x8 *)(kb + kaddr[kk]);
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[kk], kfrag, kk == 0 ? zero16 : s, 0, 0, 0);
            }
        };
        // this lane's share (16 of the wave's 32 rows) of the probabilities of key j0 + n
        auto half_sum = [&](const float (&c)[4]) { return (c[0] + c[1]) + (c[2] + c[3]); };
        auto col_sum = [&](const f32x16 &s, const int j0) {
            float c[4] = {0.f, 0.f, 0.f, 0.f};
            if (j0 + 31 > wave_lim_min) {          // the block touches the diagonal (or the end of K)
                const int jj = j0 + n - delta - wave_q0 - 4 * hh;   // visible to row r iff jj <= r - 4 hh
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float pe = fast_exp2(fmaf(s[e], c2, nl[e]));
                    c[e & 3] += (jj <= 8 * (e >> 2) + (e & 3)) ? pe : 0.f;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) c[e & 3] += fast_exp2(fmaf(s[e], c2, nl[e]));
            }
            return half_sum(c);
        };
        // x0 / x1: the lane's shares for the tile's first / second 32-key block.  One half-wave swap
        // completes both sums at once: afterwards lane l holds the wave's column sum of key l of
        // the tile.  The waves' sums meet in LDS as red[tile parity][key][wave]; after the barrier
        // (which also publishes a K tile) wave it2 % NWAVES adds the NWAVES values of each key in
        // the fixed order wave 0, 1, ... and stores the tile's 64 sums.
        auto tile_done = [&](const int it2, const float x0, const float x1) {
            const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x0), __float_as_uint(x1), false, false);
            red[(((it2 & 1) * 64 + lane) * NWAVES) + wave] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
            // every step requests one tile (NLD loads per wave): all but the two youngest requests
            // have landed, i.e. the tiles up to it2 + 3; a store of the summing wave in between
            // only makes the wait stricter
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" : : "n"(2 * NLD) : "memory");
            __syncthreads();
            if (wave == it2 % NWAVES) {
                f32x4 v[NWAVES / 4];
#pragma unroll
                for (int q = 0; q < NWAVES / 4; ++q)
                    v[q] = *(const f32x4 *)(red + (((it2 & 1) * 64 + lane) * NWAVES) + 4 * q);
                float acc = v[0][0];
#pragma unroll
                for (int w = 1; w < NWAVES; ++w) acc += v[w / 4][w % 4];
                const int j = 64 * it2 + lane;
                if (j < nk) part_row[j] = acc;
            }
        };
        // At the top of step it2 the scores of tile it2 are in registers, tiles it2+1 and it2+2 are
        // in LDS (tile t in buffer t % kSweepBufs) and tiles it2+3, it2+4 are requested.
        f32x16 sa[2] = {zero16, zero16}, sb[2] = {zero16, zero16};
        if (n_tiles > 0) {
            qk_rows(0, sa[0]);
            qk_rows(32 * ROWB, sa[1]);
        }
        int it2 = 0;
        // Tiles every row of the workgroup sees in full and that have a successor (the same ones as
        // in the first sweep): no masks.  While the probabilities of tile it2 are summed, the 16
        // MFMAs of tile it2+1 are issued, alternating between its two 32-key blocks so that
        // consecutive MFMAs are independent; each K fragment is read four MFMAs before its use.
        bf16x8 fr[4];
        auto frag_at = [&](uint32_t tile_off, int i) {
            return *(const bf16x8 *)(Ks + tile_off + (i & 1) * 32 * ROWB + kaddr[i >> 1]);
        };
        auto sweep_step = [&](auto par_c, const f32x16 (&sc)[2], f32x16 (&sn)[2]) __attribute__((always_inline)) {
            constexpr int PAR = decltype(par_c)::value;      // it2 % kSweepBufs
            constexpr uint32_t T1 = (uint32_t)((PAR + 1) % kSweepBufs) * kTileBytes;
            constexpr uint32_t T2 = (uint32_t)((PAR + 2) % kSweepBufs) * kTileBytes;
            issue_k(it2 + kSweepAhead, (PAR + kSweepAhead) % kSweepBufs);
            constexpr int NM = 2 * NKK;                      // MFMAs of a tile
            constexpr int EP = 32 / NM;                      // probabilities summed per MFMA
            float c[2][4];
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                const int blk = i & 1, kk = i >> 1;
                sn[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[kk], fr[i & 3], kk == 0 ? zero16 : sn[blk], 0, 0, 0);
                fr[i & 3] = i + 4 < NM ? frag_at(T1, i + 4) : frag_at(T2, i + 4 - NM);
#pragma unroll
                for (int x = 0; x < EP; ++x) {
                    const int cb = i / NKK, e = EP * (i % NKK) + x;
                    const float pe = fast_exp2(fmaf(sc[cb][e], c2, nl[e]));
                    c[cb][e & 3] = e < 4 ? pe : c[cb][e & 3] + pe;
                }
            }
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // 1 MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);    // 1 DS read
                __builtin_amdgcn_sched_group_barrier(0x002, EP, 0);   // multiply-adds
                __builtin_amdgcn_sched_group_barrier(0x400, EP, 0);   // transcendental
                __builtin_amdgcn_sched_group_barrier(0x002, EP, 0);   // additions
            }
            tile_done(it2, half_sum(c[0]), half_sum(c[1]));
            ++it2;
        };
        if (n_hot > 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) fr[i] = frag_at(kTileBytes, i);
            while (it2 + 6 <= n_hot) {
                sweep_step(std::integral_constant<int, 0>{}, sa, sb);
                sweep_step(std::integral_constant<int, 1>{}, sb, sa);
                sweep_step(std::integral_constant<int, 2>{}, sa, sb);
                sweep_step(std::integral_constant<int, 3>{}, sb, sa);
                sweep_step(std::integral_constant<int, 4>{}, sa, sb);
                sweep_step(std::integral_constant<int, 5>{}, sb, sa);
            }
            if (it2 < n_hot) sweep_step(std::integral_constant<int, 0>{}, sa, sb);
            if (it2 < n_hot) sweep_step(std::integral_constant<int, 1>{}, sb, sa);
            if (it2 < n_hot) sweep_step(std::integral_constant<int, 2>{}, sa, sb);
            if (it2 < n_hot) sweep_step(std::integral_constant<int, 3>{}, sb, sa);
            if (it2 < n_hot) sweep_step(std::integral_constant<int, 4>{}, sa, sb);
            if (n_hot & 1) { sa[0] = sb[0]; sa[1] = sb[1]; }
        }
        // the diagonal region; sa holds the scores of its first tile
        for (; it2 < n_tiles; ++it2) {
            issue_k(it2 + kSweepAhead, (it2 + kSweepAhead) % kSweepBufs);
            const float c0 = col_sum(sa[0], 64 * it2);
            const float c1 = col_sum(sa[1], 64 * it2 + 32);
            tile_done(it2, c0, c1);
            if (it2 + 1 < n_tiles) {
                const uint32_t b1 = (uint32_t)((it2 + 1) % kSweepBufs) * kTileBytes;
                qk_rows(b1, sa[0]);
                qk_rows(b1 + 32 * ROWB, sa[1]);
            }
        }
        __builtin_amdgcn_s_waitcnt(0);   // requests past the last tile are still in flight
        // keys that no query of this tile can see
        for (int j = 64 * n_tiles + tid; j < nk; j += NWAVES * 64) part_row[j] = 0.f;
    }
#else
    (void)p;
#endif
}

}  // namespace pdd
