// C ABI of libpdd (declared in include/pdd.h): host-side argument validation
// and kernel launches.  No device memory is allocated or freed here and no
// device data is read from the host.
#include "../../include/pdd.h"

#include <hip/hip_runtime.h>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "attn_fwd.hpp"
#include "importance.hpp"
#include "select_topk.hpp"
#include "pack_mask.hpp"
#include "select_sentences.hpp"
#include "aggregate.hpp"
#include <mutex>

// Scratch of the allocation-free entry point: one copy per GPU the library runs on, held until
// the process ends.  In host code this name is only a handle for hipGetSymbolAddress; the address
// that kernels and memory calls use is the one that call returns for the current device.
#define PDD_STATIC_SCRATCH_BYTES (16u << 20)
static __device__ __align__(256) unsigned char scratch[PDD_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[512] = "";
std::atomic<int> g_attn_waves{0};  // 0 = choose per problem
std::atomic<int> g_imp_keys{0};    // keys per importance workgroup, 0 = choose per problem

pdd_status fail(pdd_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

pdd_status check_cu_host(const char *what, const int32_t *cu, int B, int total, int max_len)
{
    if (!cu) return PDD_OK;
    if (cu[0] != 0) return fail(PDD_ERR_INVALID_ARG, "%s[0] must be 0", what);
    for (int b = 0; b < B; ++b) {
        if (cu[b + 1] < cu[b]) return fail(PDD_ERR_INVALID_ARG, "%s is not non-decreasing at %d", what, b);
        if (cu[b + 1] - cu[b] > max_len)
            return fail(PDD_ERR_INVALID_ARG, "%s: sequence %d longer than max_seqlen (%d > %d)", what, b,
                        cu[b + 1] - cu[b], max_len);
    }
    if (cu[B] != total) return fail(PDD_ERR_INVALID_ARG, "%s[B] = %d differs from the total %d", what, cu[B], total);
    return PDD_OK;
}

enum Mode { MODE_PREFILL, MODE_CHUNKED, MODE_IMPORTANCE };

pdd_status check_desc(const pdd_attn_desc *d, Mode mode)
{
    if (!d) return fail(PDD_ERR_INVALID_ARG, "desc is NULL");
    if (d->batch < 1) return fail(PDD_ERR_INVALID_ARG, "batch must be >= 1");
    if (d->n_q_heads < 1 || d->n_kv_heads < 1) return fail(PDD_ERR_INVALID_ARG, "head counts must be >= 1");
    if (d->n_q_heads % d->n_kv_heads) return fail(PDD_ERR_INVALID_ARG, "n_q_heads %% n_kv_heads != 0");
    if (d->head_dim != 64 && d->head_dim != 128)
        return fail(PDD_ERR_UNSUPPORTED, "head_dim %d not supported (64 or 128)", d->head_dim);
    if (d->total_q < 0 || d->total_k < 0) return fail(PDD_ERR_INVALID_ARG, "negative totals");
    if (d->max_seqlen_q < 0 || d->max_seqlen_k < 0 || d->max_seqlen_q > d->total_q || d->max_seqlen_k > d->total_k)
        return fail(PDD_ERR_INVALID_ARG, "max_seqlen out of range");
    if (d->total_q > 0 && d->max_seqlen_q < 1) return fail(PDD_ERR_INVALID_ARG, "max_seqlen_q must be >= 1");
    if (d->total_k > 0 && d->max_seqlen_k < 1) return fail(PDD_ERR_INVALID_ARG, "max_seqlen_k must be >= 1");
    if (!d->cu_seqlens_q || !d->cu_seqlens_k) return fail(PDD_ERR_INVALID_ARG, "cu_seqlens pointers are NULL");
    if (mode == MODE_PREFILL && d->total_q != d->total_k)
        return fail(PDD_ERR_INVALID_ARG, "prefill needs total_q == total_k (use the chunked entry point)");
    if (d->total_k < d->total_q) return fail(PDD_ERR_INVALID_ARG, "total_k < total_q");
    const int64_t hd = d->head_dim;
    const int64_t st[8] = {d->q_stride_tok, d->q_stride_head, d->k_stride_tok, d->k_stride_head,
                           d->v_stride_tok, d->v_stride_head, d->o_stride_tok, d->o_stride_head};
    const int n_st = mode == MODE_IMPORTANCE ? 4 : 8;
    for (int i = 0; i < n_st; ++i) {
        if (st[i] < hd) return fail(PDD_ERR_INVALID_ARG, "stride %d smaller than head_dim", i);
        if (st[i] % 8) return fail(PDD_ERR_INVALID_ARG, "stride %d is not a multiple of 8 elements (16 bytes)", i);
    }
    if (mode == MODE_PREFILL && d->window < 0) return fail(PDD_ERR_INVALID_ARG, "window must be >= 0");
    if (mode == MODE_IMPORTANCE && d->window == 0) return fail(PDD_ERR_INVALID_ARG, "window must not be 0");
    pdd_status s = check_cu_host("cu_seqlens_q_host", d->cu_seqlens_q_host, d->batch, d->total_q, d->max_seqlen_q);
    if (s) return s;
    s = check_cu_host("cu_seqlens_k_host", d->cu_seqlens_k_host, d->batch, d->total_k, d->max_seqlen_k);
    if (s) return s;
    if (d->cu_seqlens_q_host && d->cu_seqlens_k_host) {
        for (int b = 0; b < d->batch; ++b) {
            const int nq = d->cu_seqlens_q_host[b + 1] - d->cu_seqlens_q_host[b];
            const int nk = d->cu_seqlens_k_host[b + 1] - d->cu_seqlens_k_host[b];
            if (nk < nq) return fail(PDD_ERR_INVALID_ARG, "sequence %d has fewer keys than queries", b);
            if (mode == MODE_PREFILL && nk != nq)
                return fail(PDD_ERR_INVALID_ARG, "sequence %d: prefill needs Nq == Nk", b);
        }
    }
    return PDD_OK;
}

float scale_log2(const pdd_attn_desc *d)
{
    const float s = d->softmax_scale > 0.f ? d->softmax_scale : 1.0f / std::sqrt((float)d->head_dim);
    return s * 1.4426950408889634f;
}

// The dynamic-LDS limit of a kernel is raised once per (kernel, device), not on every launch.
pdd_status raise_lds_limit(const void *kern, int bytes)
{
    struct Done { const void *kern; int dev; };
    static Done done[64];
    static int n_done = 0;
    static std::mutex mu;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(PDD_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < n_done; ++i)
        if (done[i].kern == kern && done[i].dev == dev) return PDD_OK;
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return fail(PDD_ERR_HIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
    if (n_done < 64) done[n_done++] = {kern, dev};
    return PDD_OK;
}

template <typename Kern>
pdd_status launch_attn_kernel(Kern kern, int smem, int threads, const pdd::AttnParams &p, int64_t blocks,
                              hipStream_t st)
{
    const pdd_status s = raise_lds_limit(reinterpret_cast<const void *>(kern), smem);
    if (s) return s;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(threads), smem, st, p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(PDD_ERR_HIP, "attention launch: %s", hipGetErrorString(e));
    return PDD_OK;
}

template <int D, int NW>
pdd_status launch_attn_t(const pdd::AttnParams &p, int64_t blocks, hipStream_t st)
{
    if (p.imp_part)
        return launch_attn_kernel(pdd::attn_fwd_kernel<D, NW, true>, pdd::AttnSmem<D>::SWEEP_BYTES, NW * 64, p, blocks, st);
    return launch_attn_kernel(pdd::attn_fwd_kernel<D, NW>, pdd::AttnSmem<D>::BYTES, NW * 64, p, blocks, st);
}

int compute_units();

// Queries per attention workgroup.  8 waves (256 queries, one workgroup per compute unit) halve the
// K/V traffic into LDS per flop and win wherever the compute units stay evenly busy; 4 waves (128
// queries: twice as many workgroups of half the rows, which spread more evenly; at head_dim 64
// two of them also share a compute unit) win on small grids.  Measured on 256 compute units, T = number of 256-query tiles:
// chunks behind a prefix at least as long (workgroups of nearly equal length) prefer 8 waves from
// T = 192 on (1.0 against 0.8 PFLOP/s) and 4 waves at T = 128 (0.87 against 0.76); causal prefill,
// whose workgroups differ in length by the number of query tiles, needs more than one 8-wave
// workgroup per compute unit before their dynamic placement evens out: 4 waves up to T = 256
// (0.76 against 0.70 PFLOP/s at 4096 tokens x 16 heads), 8 waves from T = 288 on.
int attn_rows_per_workgroup(const pdd_attn_desc *d)
{
    int nw = g_attn_waves;
    if (nw == 0) {
        const int64_t tiles256 = (int64_t)((d->max_seqlen_q + 255) / 256) * d->batch * d->n_q_heads;
        const bool even_lengths = d->max_seqlen_k - d->max_seqlen_q >= d->max_seqlen_q;
        const int64_t cus = compute_units();
        nw = tiles256 > (even_lengths ? cus / 2 : cus) ? 8 : 4;
    }
    return nw * 32;
}

// Chunked mode can take the token importance from a second sweep inside the
// attention kernel (every query of the call is a window query there).  Its partial sums need one
// float per (query head, query tile, key); 0 = this shape does not use the sweep.
constexpr size_t kSweepWorkspaceMax = (size_t)256 << 20;
size_t sweep_workspace(const pdd_attn_desc *d)
{
    if (d->total_q == 0 || d->total_k == 0) return 0;
    const int bm = attn_rows_per_workgroup(d);
    const size_t n_qtiles = (size_t)((d->max_seqlen_q + bm - 1) / bm);
    // The sweep costs what full query tiles cost, the separate kernel what the rows present
    // cost: chunks that fill their tiles to less than 70 % take the separate kernel (measured on
    // 4 x (q + 8192) x 64 heads, sweep against separate kernel: 335 / 348 us at q = 192,
    // 327 / 301 at q = 160, 287 / 168 at q = 64).
    if (10 * (int64_t)d->max_seqlen_q < 7 * (int64_t)n_qtiles * bm) return 0;
    const size_t need = n_qtiles * d->n_q_heads * (size_t)d->total_k * sizeof(float);
    return need <= kSweepWorkspaceMax ? need : 0;
}

void launch_importance_reduce(const float *part, float *imp, int64_t n, int n_split, hipStream_t st)
{
    hipLaunchKernelGGL(pdd::importance_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                       part, imp, n, n_split);
}

// imp_part != NULL: sweep_workspace(d) bytes; the importance sweep runs inside
// the attention kernel and leaves its partial sums there.
pdd_status launch_attn(const pdd_attn_desc *d, const void *q, const void *k, const void *v, void *o, float *lse,
                       hipStream_t st, float *imp_part = nullptr)
{
    if (d->total_q == 0) return PDD_OK;
    pdd::AttnParams p;
    p.imp_part = imp_part;
    p.q = (const uint16_t *)q;  p.k = (const uint16_t *)k;  p.v = (const uint16_t *)v;
    p.o = (uint16_t *)o;  p.lse = lse;
    p.cu_q = d->cu_seqlens_q;  p.cu_k = d->cu_seqlens_k;
    p.q_st = d->q_stride_tok;  p.q_sh = d->q_stride_head;
    p.k_st = d->k_stride_tok;  p.k_sh = d->k_stride_head;
    p.v_st = d->v_stride_tok;  p.v_sh = d->v_stride_head;
    p.o_st = d->o_stride_tok;  p.o_sh = d->o_stride_head;
    p.B = d->batch;  p.Hq = d->n_q_heads;  p.Hkv = d->n_kv_heads;  p.G = d->n_q_heads / d->n_kv_heads;
    p.total_q = d->total_q;  p.total_k = d->total_k;
    p.scale_log2 = scale_log2(d);

    const int bm = attn_rows_per_workgroup(d);
    const int nw = bm / 32;
    p.n_qtiles = (d->max_seqlen_q + bm - 1) / bm;
    const int64_t blocks = (int64_t)p.n_qtiles * d->batch * d->n_q_heads;
    if (blocks > 0x7fffffffLL) return fail(PDD_ERR_INVALID_ARG, "launch grid too large");
    {   // 32-bit byte offsets inside one sequence's K / V span (buffer addressing); the kernels
        // request up to six tiles of 64 rows past a sequence's end, which read as zero
        const int64_t span = ((int64_t)d->max_seqlen_k + 512) * 2 *
                             (d->k_stride_tok > d->v_stride_tok ? d->k_stride_tok : d->v_stride_tok);
        if (span >= (1LL << 32)) return fail(PDD_ERR_UNSUPPORTED, "a sequence's K/V span must stay below 4 GiB");
        // and inside the 32 query rows of a wave
        if ((int64_t)d->q_stride_tok * 2 * 32 >= (1LL << 32))
            return fail(PDD_ERR_UNSUPPORTED, "32 rows of Q must span less than 4 GiB");
    }
    if (d->head_dim == 128)
        return nw == 8 ? launch_attn_t<128, 8>(p, blocks, st) : launch_attn_t<128, 4>(p, blocks, st);
    return nw == 8 ? launch_attn_t<64, 8>(p, blocks, st) : launch_attn_t<64, 4>(p, blocks, st);
}

template <int QPT>
void launch_select_reg(const pdd::SelParams &p, dim3 grid, hipStream_t st)
{
    if (p.pool_r == 0)
        hipLaunchKernelGGL((pdd::select_topk_reg_kernel<QPT, false>), grid, dim3(pdd::kSelThreads), 0, st, p);
    else
        hipLaunchKernelGGL((pdd::select_topk_reg_kernel<QPT, true>), grid, dim3(pdd::kSelThreads), 0, st, p);
}

int compute_units()
{
    static std::atomic<int> cached{0};
    int n = cached.load();
    if (n > 0) return n;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
        return 256;                       // no device visible (host-only use): the MI355X figure
    cached.store(n);
    return n;
}

// Into how many workgroups the window rows of one 256-key slice are divided.  The importance
// kernel runs three 4-wave workgroups per compute unit; with one workgroup per slice the last
// round of a launch is often mostly empty and every workgroup walks all of its row blocks alone.
// The choice minimises rounds x (row blocks per workgroup + a start-up cost of about six row
// blocks), charges the extra reduction pass as three more, and only leaves the single-pass form
// for a gain above 15 % (measured: 246 -> 220 us on 4 x 8448 keys x 64 heads x 256 rows, nothing
// on the 32k-token prompt with its 128 window rows).  It depends only on the descriptor and the
// device.
int importance_split(const pdd_attn_desc *d, int window)
{
    const int64_t slots = 3 * (int64_t)compute_units();
    const int64_t n_ktiles = (d->max_seqlen_k + pdd::kImpBK - 1) / pdd::kImpBK;
    const int64_t wgs = n_ktiles * d->batch * d->n_kv_heads;
    const int w = (window < 0 || window > d->max_seqlen_q) ? d->max_seqlen_q : window;
    const int64_t items = (int64_t)(d->n_q_heads / d->n_kv_heads) * ((w + 31) / 32);
    auto cost = [&](int r) {
        const double rounds = (double)((wgs * r + slots - 1) / slots);
        return rounds * ((double)((items + r - 1) / r) + 6.0) + (r > 1 ? 3.0 : 0.0);
    };
    int best = 1;
    for (int r = 2; r <= 8 && items / r >= 4; ++r)
        if (cost(r) < (best == 1 ? 0.85 * cost(1) : cost(best))) best = r;
    return best;
}

size_t importance_workspace(const pdd_attn_desc *d, int window)
{
    const int r = importance_split(d, window);
    return r > 1 ? (size_t)r * d->n_kv_heads * (size_t)d->total_k * sizeof(float) : 0;
}

pdd_status launch_importance(const pdd_attn_desc *d, const void *q, const void *k, const float *lse, float *imp,
                             int window, void *workspace, size_t workspace_bytes, hipStream_t st)
{
    if (d->total_k == 0) return PDD_OK;
    pdd::ImpParams p;
    p.q = (const uint16_t *)q;  p.k = (const uint16_t *)k;  p.lse = lse;  p.imp = imp;
    p.cu_q = d->cu_seqlens_q;  p.cu_k = d->cu_seqlens_k;
    p.q_st = d->q_stride_tok;  p.q_sh = d->q_stride_head;
    p.k_st = d->k_stride_tok;  p.k_sh = d->k_stride_head;
    p.B = d->batch;  p.Hq = d->n_q_heads;  p.Hkv = d->n_kv_heads;  p.G = d->n_q_heads / d->n_kv_heads;
    p.total_q = d->total_q;  p.total_k = d->total_k;
    p.window = window;
    p.scale_log2 = scale_log2(d);
    p.n_ktiles = (d->max_seqlen_k + pdd::kImpBK - 1) / pdd::kImpBK;
    {   // 32-bit byte offsets inside one sequence's Q rows (buffer addressing)
        const int64_t span = 2 * ((int64_t)d->max_seqlen_q * d->q_stride_tok + (int64_t)d->n_q_heads * d->q_stride_head);
        if (span >= (1LL << 32)) return fail(PDD_ERR_UNSUPPORTED, "a sequence's Q span must stay below 4 GiB");
        if ((int64_t)d->n_q_heads * d->total_q * 4 >= (1LL << 32))
            return fail(PDD_ERR_UNSUPPORTED, "the log-sum-exp tensor must stay below 4 GiB");
    }
    // the row split needs room for its partial sums; without it the single-pass form runs
    const size_t need = importance_workspace(d, window);
    const bool split = need > 0 && workspace && workspace_bytes >= need;
    if (split && (reinterpret_cast<uintptr_t>(workspace) & 15u))
        return fail(PDD_ERR_WORKSPACE, "workspace must be 16-byte aligned");
    p.n_split = split ? importance_split(d, window) : 1;
    p.part = split ? (float *)workspace : nullptr;
    int64_t blocks = (int64_t)p.n_ktiles * d->batch * d->n_kv_heads * p.n_split;
    // Up to four workgroups per compute unit the launch runs with half the keys per workgroup
    // (one 32-key group per wave instead of two): the same blocks of rows per workgroup at half
    // the work per block, and a workgroup's time is mostly its chain of blocks.  Measured against
    // 256 keys: 17 -> 12 us on 4096 tokens x 32 heads (128 workgroups become 256), 42 -> 37 us on
    // the batch of 8 mixed prompts (768 -> 1536), equal on the 32k-token prompt (1024 -> 2048);
    // beyond that the wide form re-reads the window rows half as often.  Same bits either way.
    // (Counted in workgroups that have keys: the grid is sized for the longest sequence.)
    const int64_t working = (int64_t)d->total_k / pdd::kImpBK * d->n_kv_heads * p.n_split;
    const bool narrow = g_imp_keys ? g_imp_keys == pdd::kImpBK / 2 : working <= 4 * (int64_t)compute_units();
    if (narrow) {
        p.n_ktiles = (d->max_seqlen_k + pdd::kImpBK / 2 - 1) / (pdd::kImpBK / 2);
        blocks = (int64_t)p.n_ktiles * d->batch * d->n_kv_heads * p.n_split;
    }
    if (blocks > 0x7fffffffLL) return fail(PDD_ERR_INVALID_ARG, "launch grid too large");
    const dim3 grid((unsigned)blocks), block(pdd::kImpWaves * 64);
    if (d->head_dim == 128) {
        if (narrow) hipLaunchKernelGGL((pdd::importance_kernel<128, 1>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((pdd::importance_kernel<128, 2>), grid, block, 0, st, p);
    } else {
        if (narrow) hipLaunchKernelGGL((pdd::importance_kernel<64, 1>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((pdd::importance_kernel<64, 2>), grid, block, 0, st, p);
    }
    if (split) launch_importance_reduce(p.part, imp, (int64_t)d->n_kv_heads * d->total_k, p.n_split, st);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(PDD_ERR_HIP, "importance launch: %s", hipGetErrorString(e));
    return PDD_OK;
}

// What the chunked call can use: room for the in-kernel sweep where that applies, else for the
// row split of the separate importance kernel.
size_t chunked_workspace(const pdd_attn_desc *d)
{
    const size_t sweep = sweep_workspace(d);
    return sweep ? sweep : importance_workspace(d, -1);
}

// Device address of this GPU's copy of `scratch`, looked up once per device.
pdd_status static_scratch(void **out)
{
    static void *ptr[64];
    static bool known[64];
    static std::mutex mu;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(PDD_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= 64) return fail(PDD_ERR_UNSUPPORTED, "device ordinal %d beyond 63", dev);
    std::lock_guard<std::mutex> lock(mu);
    if (!known[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(PDD_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        ptr[dev] = p;
        known[dev] = true;
    }
    *out = ptr[dev];
    return PDD_OK;
}

pdd_status check_ptrs(const void *q, const void *k, const void *v, const void *o, const void *lse)
{
    if (!q || !k || !v || !o || !lse) return fail(PDD_ERR_INVALID_ARG, "NULL tensor pointer");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o))
        return fail(PDD_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (reinterpret_cast<uintptr_t>(lse) & 3u) return fail(PDD_ERR_INVALID_ARG, "lse must be 4-byte aligned");
    return PDD_OK;
}

}  // namespace

extern "C" {

const char *pdd_last_error(void) { return g_err; }
const char *pdd_version(void) { return "pdd 0.1 gfx950"; }

pdd_status pdd_set_option(int option, int value)
{
    if (option == PDD_OPT_ATTN_WAVES) {
        if (value != 0 && value != 4 && value != 8) return fail(PDD_ERR_INVALID_ARG, "attn waves must be 0, 4 or 8");
        g_attn_waves = value;
        return PDD_OK;
    }
    if (option == PDD_OPT_IMPORTANCE_KEYS) {
        if (value != 0 && value != pdd::kImpBK / 2 && value != pdd::kImpBK)
            return fail(PDD_ERR_INVALID_ARG, "importance keys per workgroup must be 0, 128 or 256");
        g_imp_keys = value;
        return PDD_OK;
    }
    return fail(PDD_ERR_INVALID_ARG, "unknown option %d", option);
}

size_t pdd_workspace_bytes(const pdd_attn_desc *desc, int which_call)
{
    if (!desc || desc->batch < 1 || desc->n_kv_heads < 1 || desc->n_q_heads < desc->n_kv_heads || desc->total_k < 0)
        return 0;
    switch (which_call) {
    case PDD_CALL_PREFILL_ATTN:
        return desc->window > 0 ? importance_workspace(desc, desc->window) : 0;
    case PDD_CALL_PREFILL_ATTN_CHUNKED:
        return chunked_workspace(desc);
    case PDD_CALL_TOKEN_IMPORTANCE:
        return desc->window != 0 ? importance_workspace(desc, desc->window) : 0;
    default:
        return 0;  // the selection keeps its intermediates in registers / LDS
    }
}

pdd_status pdd_prefill_attn(const pdd_attn_desc *desc, const void *q, const void *k, const void *v, void *o,
                            float *lse, float *importance, void *workspace, size_t workspace_bytes,
                            pdd_stream stream)
{
    pdd_status s = check_desc(desc, MODE_PREFILL);
    if (s) return s;
    s = check_ptrs(q, k, v, o, lse);
    if (s) return s;
    if (desc->window > 0 && !importance)
        return fail(PDD_ERR_INVALID_ARG, "window > 0 needs an importance buffer");
    s = launch_attn(desc, q, k, v, o, lse, (hipStream_t)stream);
    if (s) return s;
    if (importance && desc->window > 0)
        return launch_importance(desc, q, k, lse, importance, desc->window, workspace, workspace_bytes,
                                 (hipStream_t)stream);
    return PDD_OK;
}

pdd_status pdd_prefill_attn_chunked(const pdd_attn_desc *desc, const void *q_chunk, const void *k_all,
                                    const void *v_all, void *o, float *lse, float *importance, void *workspace,
                                    size_t workspace_bytes, pdd_stream stream)
{
    pdd_status s = check_desc(desc, MODE_CHUNKED);
    if (s) return s;
    s = check_ptrs(q_chunk, k_all, v_all, o, lse);
    if (s) return s;
    const size_t sweep = importance ? sweep_workspace(desc) : 0;
    if (sweep && workspace && workspace_bytes >= sweep) {
        if (reinterpret_cast<uintptr_t>(workspace) & 15u)
            return fail(PDD_ERR_WORKSPACE, "workspace must be 16-byte aligned");
        s = launch_attn(desc, q_chunk, k_all, v_all, o, lse, (hipStream_t)stream, (float *)workspace);
        if (s) return s;
        const int bm = attn_rows_per_workgroup(desc);
        const int n_slices = (desc->n_q_heads / desc->n_kv_heads) * ((desc->max_seqlen_q + bm - 1) / bm);
        launch_importance_reduce((const float *)workspace, importance, (int64_t)desc->n_kv_heads * desc->total_k,
                                 n_slices, (hipStream_t)stream);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(PDD_ERR_HIP, "importance reduction launch: %s", hipGetErrorString(e));
        return PDD_OK;
    }
    s = launch_attn(desc, q_chunk, k_all, v_all, o, lse, (hipStream_t)stream);
    if (s) return s;
    if (importance)
        return launch_importance(desc, q_chunk, k_all, lse, importance, -1, workspace, workspace_bytes,
                                 (hipStream_t)stream);
    return PDD_OK;
}

pdd_status pdd_prefill_attn_chunked_noalloc(const pdd_attn_desc *desc, const void *q_chunk, const void *k_all,
                                            const void *v_all, void *o, float *lse, float *importance,
                                            pdd_stream stream)
{
    pdd_status s = check_desc(desc, MODE_CHUNKED);
    if (s) return s;
    const size_t need = importance ? chunked_workspace(desc) : 0;
    if (need > PDD_STATIC_SCRATCH_BYTES)
        return fail(PDD_ERR_WORKSPACE, "this shape wants %zu bytes of scratch, the built-in scratch holds %u "
                    "(use pdd_prefill_attn_chunked with a workspace)", need, (unsigned)PDD_STATIC_SCRATCH_BYTES);
    void *ws = nullptr;
    if (need > 0) {
        s = static_scratch(&ws);
        if (s) return s;
    }
    return pdd_prefill_attn_chunked(desc, q_chunk, k_all, v_all, o, lse, importance, ws, need, stream);
}

pdd_status pdd_token_importance(const pdd_attn_desc *desc, const void *q, const void *k, const float *lse,
                                float *importance, void *workspace, size_t workspace_bytes, pdd_stream stream)
{
    pdd_status s = check_desc(desc, MODE_IMPORTANCE);
    if (s) return s;
    if (!q || !k || !lse || !importance) return fail(PDD_ERR_INVALID_ARG, "NULL tensor pointer");
    if (!aligned16(q) || !aligned16(k)) return fail(PDD_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    return launch_importance(desc, q, k, lse, importance, desc->window, workspace, workspace_bytes,
                             (hipStream_t)stream);
}

pdd_status pdd_select_topk_pooled(const float *scores, int32_t n_heads, int32_t batch, int32_t total_k,
                                  const int32_t *cu_seqlens_k, const int32_t *cu_seqlens_k_host,
                                  int32_t max_seqlen_k, const int32_t *cand_begin, const int32_t *cand_end,
                                  const int32_t *k_per_seq, const int32_t *cu_keep, int32_t total_keep,
                                  int32_t pool_kernel, int32_t pool_mode, float *pooled_out,
                                  int32_t *out_indices, uint8_t *out_mask, void *workspace,
                                  size_t workspace_bytes, pdd_stream stream)
{
    (void)workspace;
    (void)workspace_bytes;
    if (!scores || !cu_seqlens_k || !k_per_seq || !cu_keep) return fail(PDD_ERR_INVALID_ARG, "NULL pointer");
    if (n_heads < 1 || batch < 1) return fail(PDD_ERR_INVALID_ARG, "n_heads and batch must be >= 1");
    if (total_k < 0 || total_keep < 0 || max_seqlen_k < 0 || max_seqlen_k > total_k)
        return fail(PDD_ERR_INVALID_ARG, "bad sizes");
    if (total_keep > 0 && !out_indices) return fail(PDD_ERR_INVALID_ARG, "out_indices is NULL");
    if ((cand_begin == nullptr) != (cand_end == nullptr))
        return fail(PDD_ERR_INVALID_ARG, "cand_begin and cand_end must both be given or both be NULL");
    if (batch > 65535 * 32) return fail(PDD_ERR_INVALID_ARG, "batch too large");
    if (n_heads > 65535) return fail(PDD_ERR_INVALID_ARG, "n_heads too large");
    if (pool_mode != PDD_POOL_NONE && pool_mode != PDD_POOL_MAX && pool_mode != PDD_POOL_AVG)
        return fail(PDD_ERR_INVALID_ARG, "unknown pool_mode %d", pool_mode);
    if (pool_mode != PDD_POOL_NONE && (pool_kernel < 1 || pool_kernel % 2 == 0 || pool_kernel > 1025))
        return fail(PDD_ERR_INVALID_ARG, "pool_kernel must be odd and in [1, 1025]");
    pdd_status s = check_cu_host("cu_seqlens_k_host", cu_seqlens_k_host, batch, total_k, max_seqlen_k);
    if (s) return s;
    if (total_k == 0) return PDD_OK;

    pdd::SelParams p;
    p.scores = scores;  p.cu_k = cu_seqlens_k;  p.cand_b = cand_begin;  p.cand_e = cand_end;
    p.k_per = k_per_seq;  p.cu_keep = cu_keep;  p.out_idx = out_indices;  p.out_mask = out_mask;
    p.n_heads = n_heads;  p.B = batch;  p.total_k = total_k;  p.total_keep = total_keep;
    p.pool_r = pool_mode == PDD_POOL_NONE ? 0 : (pool_kernel - 1) / 2;
    p.pool_mode = pool_mode == PDD_POOL_MAX ? pdd::kPoolMax : pdd::kPoolAvg;
    p.pool_inv = pool_mode == PDD_POOL_AVG ? 1.0f / (float)pool_kernel : 1.0f;
    p.pooled_out = pooled_out;
    const dim3 grid((unsigned)batch, (unsigned)n_heads);
    hipStream_t st = (hipStream_t)stream;
    // rows of up to 32768 candidates stay in registers (4096 per step and 1024 threads)
    if (max_seqlen_k <= 4 * pdd::kSelThreads)
        launch_select_reg<1>(p, grid, st);
    else if (max_seqlen_k <= 8 * pdd::kSelThreads)
        launch_select_reg<2>(p, grid, st);
    else if (max_seqlen_k <= 16 * pdd::kSelThreads)
        launch_select_reg<4>(p, grid, st);
    else if (max_seqlen_k <= 32 * pdd::kSelThreads)
        launch_select_reg<8>(p, grid, st);
    else
        hipLaunchKernelGGL(pdd::select_topk_kernel, grid, dim3(pdd::kSelThreads), 0, st, p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(PDD_ERR_HIP, "select launch: %s", hipGetErrorString(e));
    return PDD_OK;
}

pdd_status pdd_select_topk(const float *scores, int32_t n_heads, int32_t batch, int32_t total_k,
                           const int32_t *cu_seqlens_k, const int32_t *cu_seqlens_k_host, int32_t max_seqlen_k,
                           const int32_t *cand_begin, const int32_t *cand_end, const int32_t *k_per_seq,
                           const int32_t *cu_keep, int32_t total_keep, int32_t *out_indices, uint8_t *out_mask,
                           void *workspace, size_t workspace_bytes, pdd_stream stream)
{
    return pdd_select_topk_pooled(scores, n_heads, batch, total_k, cu_seqlens_k, cu_seqlens_k_host, max_seqlen_k,
                                  cand_begin, cand_end, k_per_seq, cu_keep, total_keep, 1, PDD_POOL_NONE, nullptr,
                                  out_indices, out_mask, workspace, workspace_bytes, stream);
}

pdd_status pdd_select_sentences(const float *scores, int32_t n_heads, int32_t batch, int32_t total_k,
                                const int32_t *cu_seqlens_k, const int32_t *cu_seqlens_k_host, int32_t max_seqlen_k,
                                const int32_t *cu_sent, const int32_t *sent_end, int32_t total_sent,
                                int32_t max_sent_per_seq, const int32_t *cand_begin, const int32_t *token_budget,
                                int32_t agg_mode, float *out_sent_scores, uint8_t *out_sent_keep,
                                uint8_t *out_mask, int32_t *out_kept_tokens, pdd_stream stream)
{
    if (!scores || !cu_seqlens_k || !cu_sent || !token_budget) return fail(PDD_ERR_INVALID_ARG, "NULL pointer");
    if (total_sent > 0 && !sent_end) return fail(PDD_ERR_INVALID_ARG, "sent_end is NULL");
    if (n_heads < 1 || batch < 1) return fail(PDD_ERR_INVALID_ARG, "n_heads and batch must be >= 1");
    if (total_k < 0 || total_sent < 0 || max_seqlen_k < 0 || max_seqlen_k > total_k || max_sent_per_seq < 0 ||
        max_sent_per_seq > total_sent)
        return fail(PDD_ERR_INVALID_ARG, "bad sizes");
    if (max_sent_per_seq > pdd::kSentMax)
        return fail(PDD_ERR_UNSUPPORTED, "more than %d sentences in one sequence", pdd::kSentMax);
    if (agg_mode != PDD_SENT_SUM && agg_mode != PDD_SENT_MEAN) return fail(PDD_ERR_INVALID_ARG, "unknown agg_mode");
    if (batch > 65535 * 32 || n_heads > 65535) return fail(PDD_ERR_INVALID_ARG, "batch or n_heads too large");
    pdd_status s = check_cu_host("cu_seqlens_k_host", cu_seqlens_k_host, batch, total_k, max_seqlen_k);
    if (s) return s;
    if (total_k == 0) return PDD_OK;
    pdd::SentParams p;
    p.scores = scores;  p.cu_k = cu_seqlens_k;  p.cu_sent = cu_sent;  p.sent_end = sent_end;
    p.cand_b = cand_begin;  p.budget = token_budget;  p.sent_keep = out_sent_keep;  p.mask = out_mask;
    p.kept_tokens = out_kept_tokens;  p.sent_scores = out_sent_scores;
    p.n_heads = n_heads;  p.B = batch;  p.total_k = total_k;  p.total_sent = total_sent;
    p.s_cap = max_sent_per_seq > 0 ? ((max_sent_per_seq + 3) & ~3) : 4;
    p.mode = agg_mode == PDD_SENT_MEAN ? pdd::kSentMean : pdd::kSentSum;
    const int smem = p.s_cap * 16;
    s = raise_lds_limit(reinterpret_cast<const void *>(pdd::select_sentences_kernel), pdd::kSentMax * 16);
    if (s) return s;
    hipError_t e;
    hipLaunchKernelGGL(pdd::select_sentences_kernel, dim3((unsigned)batch, (unsigned)n_heads),
                       dim3(pdd::kSelThreads), smem, (hipStream_t)stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) return fail(PDD_ERR_HIP, "sentence select launch: %s", hipGetErrorString(e));
    return PDD_OK;
}

pdd_status pdd_aggregate_scores(const float *scores, int32_t n_layers, int32_t n_heads, int32_t total_k,
                                int64_t layer_stride, const float *layer_weights, int32_t reduce_heads,
                                int32_t accumulate, float *out, pdd_stream stream)
{
    if (!scores || !out) return fail(PDD_ERR_INVALID_ARG, "NULL pointer");
    if (n_layers < 1 || n_heads < 1 || n_heads > 65535 || total_k < 0)
        return fail(PDD_ERR_INVALID_ARG, "bad sizes");
    if (layer_stride < (int64_t)n_heads * total_k)
        return fail(PDD_ERR_INVALID_ARG, "layer_stride smaller than n_heads * total_k");
    if (total_k == 0) return PDD_OK;
    pdd::AggParams p;
    p.scores = scores;  p.weights = layer_weights;  p.out = out;  p.layer_stride = layer_stride;
    p.n_layers = n_layers;  p.n_heads = n_heads;  p.total_k = total_k;
    p.reduce_heads = reduce_heads ? 1 : 0;  p.accumulate = accumulate ? 1 : 0;
    const bool vec = total_k % 4 == 0 && layer_stride % 4 == 0 && ((uintptr_t)scores % 16) == 0 &&
                     ((uintptr_t)out % 16) == 0;
    const int per_block = 256 * (vec ? 4 : 1);
    const dim3 grid((unsigned)((total_k + per_block - 1) / per_block), (unsigned)(reduce_heads ? 1 : n_heads));
    if (vec) hipLaunchKernelGGL(pdd::aggregate_scores_kernel<4>, grid, dim3(256), 0, (hipStream_t)stream, p);
    else     hipLaunchKernelGGL(pdd::aggregate_scores_kernel<1>, grid, dim3(256), 0, (hipStream_t)stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(PDD_ERR_HIP, "aggregate launch: %s", hipGetErrorString(e));
    return PDD_OK;
}

/* Host-only scalar code: the closed form of the program that picks (r, L). */
pdd_status pdd_choose_r_L(const pdd_rl_model *m, int32_t l, double *r_out, int32_t *L_out)
{
    if (!m || !r_out || !L_out) return fail(PDD_ERR_INVALID_ARG, "NULL pointer");
    if (l < 1) return fail(PDD_ERR_INVALID_ARG, "prompt length must be >= 1");
    if (!(m->k_c >= 0) || !(m->k_d > 0) || !(m->delta >= 0) || !(m->tpot_c > 0) || !(m->tpot_d > 0) ||
        !(m->xi_scene >= 0 && m->xi_scene <= 1))
        return fail(PDD_ERR_INVALID_ARG, "model coefficients out of range");
    if (!(m->delta_cloud >= 0 && m->delta_cloud <= m->delta))
        return fail(PDD_ERR_INVALID_ARG, "delta_cloud must lie in [0, delta]");
    if (!(m->tau > m->tpot_d)) return fail(PDD_ERR_INFEASIBLE, "tau must exceed the device TPOT");
    const double len = (double)l;
    /* In terms of x = k_d*r*l (device prefill time of the refined prompt) and n = L - 1 >= 1:
     *   Eq. 5: x_min = k_d*xi*l <= x <= x_max = k_d*l - k_c*l - delta
     *   Eq. 6: n*tpot_c - (delta - delta_cloud) <= x <= n*(tau - tpot_d) + TTFT_c
     * The objective grows with x.  Below n0 = the smallest n whose upper bound reaches x_min
     * nothing is feasible; from n0 on the lower bound only grows with n, so the optimum is
     * n0 with x = max(x_min, n0*tpot_c - decompress), if that still respects both upper bounds. */
    const double ttft_c = m->k_c * len + m->delta_cloud;          /* prefill + compress + RTT */
    const double decompress = m->delta - m->delta_cloud;
    const double a = m->tau - m->tpot_d;
    const double x_min = m->k_d * m->xi_scene * len;
    const double x_max = m->k_d * len - m->k_c * len - m->delta;
    if (x_min > x_max) return fail(PDD_ERR_INFEASIBLE, "no ratio in [xi_scene, %.6g]", x_max / (m->k_d * len));
    double n0 = std::ceil((x_min - ttft_c) / a);
    if (n0 < 1.0) n0 = 1.0;
    if (n0 > 2147483646.0) return fail(PDD_ERR_INFEASIBLE, "L out of range");
    double x = n0 * m->tpot_c - decompress;
    double r = x / (m->k_d * len);
    if (x <= x_min) { x = x_min; r = m->xi_scene; }
    if (x > x_max || x > n0 * a + ttft_c)
        return fail(PDD_ERR_INFEASIBLE, "no (r, L): L - 1 = %.0f needs a device prefill of %.6g, allowed at most %.6g",
                    n0, x, x_max < n0 * a + ttft_c ? x_max : n0 * a + ttft_c);
    const double lm1 = n0;
    *r_out = r;
    *L_out = (int32_t)lm1 + 1;
    return PDD_OK;
}

int64_t pdd_pack_mask_layout(int32_t batch, const int32_t *cu_seqlens_k_host, int32_t *cu_bytes_host)
{
    if (batch < 1 || !cu_seqlens_k_host || !cu_bytes_host) {
        fail(PDD_ERR_INVALID_ARG, "pdd_pack_mask_layout: bad arguments");
        return -1;
    }
    int64_t total = 0;
    cu_bytes_host[0] = 0;
    for (int b = 0; b < batch; ++b) {
        const int64_t nk = (int64_t)cu_seqlens_k_host[b + 1] - cu_seqlens_k_host[b];
        if (nk < 0) {
            fail(PDD_ERR_INVALID_ARG, "pdd_pack_mask_layout: cu_seqlens_k_host decreases at %d", b);
            return -1;
        }
        total += (nk + 7) / 8;
        if (total > 0x7fffffffLL) {
            fail(PDD_ERR_INVALID_ARG, "pdd_pack_mask_layout: more than 2^31 bytes per row");
            return -1;
        }
        cu_bytes_host[b + 1] = (int32_t)total;
    }
    return total;
}

pdd_status pdd_pack_mask(const uint8_t *mask, int32_t n_rows, int32_t batch, int32_t total_k,
                         const int32_t *cu_seqlens_k, const int32_t *cu_seqlens_k_host, int32_t max_seqlen_k,
                         const int32_t *cu_bytes, int32_t total_bytes, uint8_t *out_bits, pdd_stream stream)
{
    if (!mask || !cu_seqlens_k || !cu_bytes) return fail(PDD_ERR_INVALID_ARG, "NULL pointer");
    if (n_rows < 1 || batch < 1) return fail(PDD_ERR_INVALID_ARG, "n_rows and batch must be >= 1");
    if (total_k < 0 || total_bytes < 0 || max_seqlen_k < 0 || max_seqlen_k > total_k)
        return fail(PDD_ERR_INVALID_ARG, "bad sizes");
    if (total_bytes > 0 && !out_bits) return fail(PDD_ERR_INVALID_ARG, "out_bits is NULL");
    if (batch > 65535 || n_rows > 65535) return fail(PDD_ERR_INVALID_ARG, "batch or n_rows too large");
    pdd_status s = check_cu_host("cu_seqlens_k_host", cu_seqlens_k_host, batch, total_k, max_seqlen_k);
    if (s) return s;
    if (total_k == 0 || total_bytes == 0) return PDD_OK;
    pdd::PackParams p;
    p.mask = mask;  p.bits = out_bits;  p.cu_k = cu_seqlens_k;  p.cu_bytes = cu_bytes;
    p.rows = n_rows;  p.B = batch;  p.total_k = total_k;  p.total_bytes = total_bytes;
    const int max_bytes = (max_seqlen_k + 7) / 8;
    const unsigned gx = (unsigned)((max_bytes + pdd::kPackThreads - 1) / pdd::kPackThreads);
    hipLaunchKernelGGL(pdd::pack_mask_kernel, dim3(gx, (unsigned)batch, (unsigned)n_rows), dim3(pdd::kPackThreads), 0,
                       (hipStream_t)stream, p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(PDD_ERR_HIP, "pack launch: %s", hipGetErrorString(e));
    return PDD_OK;
}

}  // extern "C"
