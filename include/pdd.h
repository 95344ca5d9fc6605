/*
 * pdd.h -- C ABI of libpdd: causal prompt-prefill attention for gfx950 fused
 * with extraction of the prompt-refinement data (token importance, top-k
 * token selection).
 *
 * General conventions (all entry points)
 *   - "DEVICE" pointers are HBM addresses on the current HIP device; "HOST"
 *     pointers are ordinary process memory.  The caller owns every buffer; the
 *     library never allocates, frees or keeps a pointer after returning.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and the call returns without synchronising.  The library
 *     never reads device memory from the host.
 *   - Arguments are validated on the host before anything is launched; on a
 *     validation failure nothing has been enqueued.  The return value is the
 *     only error channel; pdd_last_error() gives a thread-local message.
 *   - Every output element that belongs to a sequence is overwritten; outputs
 *     need not be initialised.  Results are deterministic run to run.
 *   - bf16 tensors are raw 16-bit patterns; the innermost (head_dim) axis is
 *     contiguous; all DEVICE tensor pointers and all strides*2 bytes must be
 *     multiples of 16 bytes.
 *   - NaN / Inf inputs: undefined results (no fault).
 *
 * Notation: B sequences; sequence b has Nq_b queries and Nk_b >= Nq_b keys,
 * delta_b = Nk_b - Nq_b; Hq query heads, Hkv KV heads, G = Hq/Hkv; d =
 * head_dim.  Query head h reads KV head h / G.  Indices i, j are local to the
 * sequence.
 */
#ifndef PDD_H
#define PDD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum pdd_status {
    PDD_OK = 0,
    PDD_ERR_INVALID_ARG = -1, /* null pointer, bad size, Hq % Hkv != 0, misaligned, ... */
    PDD_ERR_UNSUPPORTED = -2, /* head_dim not in {64, 128}; a size beyond a documented limit */
    PDD_ERR_WORKSPACE = -3,   /* workspace smaller than pdd_workspace_bytes()           */
    PDD_ERR_HIP = -4,         /* a HIP runtime call (launch) reported an error          */
    PDD_ERR_INFEASIBLE = -5   /* pdd_choose_r_L: the constraints admit no (r, L)        */
} pdd_status;

typedef void *pdd_stream; /* hipStream_t */

/*
 * One attention layer over a packed (ragged) batch.
 *   Q, O : [total_q, Hq, d]  bf16, addressed token*stride_tok + head*stride_head + c
 *   K, V : [total_k, Hkv, d] bf16
 * Strides are in elements.  cu_seqlens_q / cu_seqlens_k are DEVICE int32
 * arrays of B+1 non-decreasing prefix sums starting at 0 and ending at
 * total_q / total_k.  The optional HOST copies (may be NULL) let the library
 * validate them (monotone, end totals, Nk_b >= Nq_b, within max_seqlen);
 * without them a malformed device array is clamped to the totals, never
 * followed out of bounds.
 */
typedef struct pdd_attn_desc {
    int32_t batch;        /* B >= 1                                            */
    int32_t n_q_heads;    /* Hq                                                */
    int32_t n_kv_heads;   /* Hkv, divides Hq                                   */
    int32_t head_dim;     /* d in {64, 128}                                    */
    int32_t total_q;      /* sum of Nq_b                                       */
    int32_t total_k;      /* sum of Nk_b                                       */
    int32_t max_seqlen_q; /* >= max Nq_b (sizes the launch grid)               */
    int32_t max_seqlen_k; /* >= max Nk_b                                       */
    const int32_t *cu_seqlens_q;      /* DEVICE int32[B+1]                     */
    const int32_t *cu_seqlens_k;      /* DEVICE int32[B+1]                     */
    const int32_t *cu_seqlens_q_host; /* HOST copy or NULL                     */
    const int32_t *cu_seqlens_k_host; /* HOST copy or NULL                     */
    int64_t q_stride_tok, q_stride_head;
    int64_t k_stride_tok, k_stride_head;
    int64_t v_stride_tok, v_stride_head;
    int64_t o_stride_tok, o_stride_head;
    float softmax_scale;  /* s; <= 0 selects 1/sqrt(d)                         */
    int32_t window;       /* W: observation window = last min(W, Nq_b) queries;
                             0 = no importance output                          */
} pdd_attn_desc;

/* which_call values for pdd_workspace_bytes */
enum {
    PDD_CALL_PREFILL_ATTN = 0,
    PDD_CALL_PREFILL_ATTN_CHUNKED = 1,
    PDD_CALL_TOKEN_IMPORTANCE = 2,
    PDD_CALL_SELECT_TOPK = 3
};

/*
 * Causal prefill attention (paper Section 2.2.3, the scaled dot-product
 * attention equation softmax(Q K^T / sqrt(h)) V with h read as the per-head
 * dimension, under the autoregressive mask), fused with the refiner's data
 * extraction (Section 3.2 "Prompt Refiner": the normalised attention weight of
 * the observation window against the entire K, summed along the query
 * dimension; Section 3.2 "Preliminaries": obtained inside the attention
 * implementation, in place, without materialising or copying the weights).
 *
 *   S[i,j]   = s * <q[i,h,:], k[j,g,:]>       for 0 <= j <= i + delta_b
 *   lse[h,i] = ln sum_j exp(S[i,j])                         (natural log)
 *   o[i,h,:] = sum_j exp(S[i,j] - lse[h,i]) * v[j,g,:]
 *   importance[g,j] = sum_{h in group g} sum_{i in window_b, i+delta_b >= j}
 *                     exp(S[i,j] - lse[h,i])
 *
 * o          DEVICE bf16 [total_q, Hq, d] (strides from desc)          -- out
 * lse        DEVICE fp32 [Hq, total_q] contiguous                      -- out
 * importance DEVICE fp32 [Hkv, total_k] contiguous, or NULL (then W is
 *            ignored); must be non-NULL when desc->window > 0          -- out
 * workspace  DEVICE scratch, 16-byte aligned, or NULL.  With at least
 *            pdd_workspace_bytes(desc, PDD_CALL_PREFILL_ATTN) bytes the
 *            importance step divides the window rows of every 256-key slice over
 *            several workgroups that leave partial column sums there, added in a
 *            fixed order afterwards; with less (or NULL) each slice is summed by
 *            one workgroup.  Both forms are deterministic; they differ from each
 *            other in the order of the fp32 additions.  The contents are
 *            scratch before and after the call; concurrent calls need separate
 *            workspaces.
 * Requires Nq_b == Nk_b for every sequence when host copies are given (use the
 * chunked entry point otherwise).
 * Limits (PDD_ERR_UNSUPPORTED beyond them; the kernels address with 32-bit byte
 * offsets): the K and V rows of one sequence,
 * (max_seqlen_k + 512) * stride_tok * 2 bytes, must span less than 4 GiB, and
 * so must 32 rows of Q (32 * q_stride_tok * 2 bytes); with
 * an importance output the same holds for one sequence's Q rows and for the
 * whole lse tensor (Hq * total_q * 4 bytes).
 */
pdd_status pdd_prefill_attn(const pdd_attn_desc *desc, const void *q, const void *k,
                            const void *v, void *o, float *lse, float *importance,
                            void *workspace, size_t workspace_bytes, pdd_stream stream);

/*
 * Chunked mode: a chunk of Nq_b new queries attends to an existing KV prefix
 * of delta_b tokens plus the chunk's own keys, causal mask aligned to the
 * bottom-right corner (the on-device engine's chunked prefill, Section 3.3
 * "LLM Engine": the prefix is processed while the first token is awaited, the
 * remaining chunk catches up afterwards).  Same formulas as above with
 * delta_b = Nk_b - Nq_b >= 0.  Every chunk query is a window query
 * (desc->window is ignored) when importance is non-NULL.
 * workspace: as for pdd_prefill_attn, with one more form.
 * Given pdd_workspace_bytes(desc, PDD_CALL_PREFILL_ATTN_CHUNKED) bytes (one
 * float per query head, tile of 128 or 256 queries and key), the importance is
 * taken inside the attention kernel: once a workgroup knows the log-sum-exp of
 * its queries it walks its K tiles a second time, with Q still in registers,
 * and leaves the column sums of its probabilities in the workspace; a short
 * second kernel adds them over the heads of a group and the query tiles in a
 * fixed order.  Shapes that would need more than 256 MiB for this, chunks
 * whose longest fills less than 70 % of its query tiles (the second walk costs
 * what full tiles cost) and calls that are given less use the separate
 * importance kernel described above; pdd_workspace_bytes says what the shape
 * will use.  All forms are deterministic and agree to fp32 rounding.
 */
pdd_status pdd_prefill_attn_chunked(const pdd_attn_desc *desc, const void *q_chunk,
                                    const void *k_all, const void *v_all, void *o, float *lse,
                                    float *importance, void *workspace, size_t workspace_bytes,
                                    pdd_stream stream);

/*
 * pdd_prefill_attn_chunked for callers that cannot allocate device memory (code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): same arguments without the workspace, same results bit for bit as
 * pdd_prefill_attn_chunked called with a workspace of pdd_workspace_bytes(desc,
 * PDD_CALL_PREFILL_ATTN_CHUNKED) bytes.  The scratch is a fixed 16 MiB array
 * inside the library's device image (one copy per GPU, held until the process
 * ends); the call allocates and frees nothing.  A shape whose scratch would
 * exceed 16 MiB is rejected with PDD_ERR_WORKSPACE and nothing is enqueued.
 * All calls on one GPU share that array: calls that overlap in time on the same
 * GPU (different streams or threads) race on it and must be serialised by the
 * caller.  Nothing in it has to be cleared between calls (every partial sum a
 * call reads it has written itself).
 */
pdd_status pdd_prefill_attn_chunked_noalloc(const pdd_attn_desc *desc, const void *q_chunk,
                                            const void *k_all, const void *v_all, void *o,
                                            float *lse, float *importance, pdd_stream stream);

/*
 * Token importance alone (Section 3.2 "Prompt Refiner"), from log-sum-exp
 * values computed earlier (e.g. by pdd_prefill_attn with importance = NULL):
 * same definition and same result as the fused output.  desc->window < 0
 * means every query is a window query; 0 is an error here.
 *   lse        DEVICE fp32 [Hq, total_q]                                -- in
 *   importance DEVICE fp32 [Hkv, total_k]                               -- out
 */
pdd_status pdd_token_importance(const pdd_attn_desc *desc, const void *q, const void *k,
                                const float *lse, float *importance, void *workspace,
                                size_t workspace_bytes, pdd_stream stream);

/*
 * Top-k token selection and stable index compaction (Section 3.2 "Prompt
 * Refiner": sort the summed scores, keep the indices with the top values per
 * head at ratio r, filter the positions; the mask tensor holds 1 at position i
 * when token i is selected).  For every KV head g and sequence b the
 * candidates are keys [cand_begin[b], cand_end[b]) of that sequence (NULL
 * arrays = the whole sequence); they are ranked by (score descending, index
 * ascending) and the first k_per_seq[b] are kept.
 *
 *   scores       DEVICE fp32 [n_heads, total_k]                          -- in
 *   cu_seqlens_k DEVICE int32[B+1]; cu_seqlens_k_host HOST copy or NULL
 *   cand_begin, cand_end DEVICE int32[B] or both NULL
 *   k_per_seq    DEVICE int32[B], 0 <= k_b <= cand_end[b]-cand_begin[b]
 *   cu_keep      DEVICE int32[B+1] prefix sums of k_per_seq
 *   total_keep   = cu_keep[B] (host copy)
 *   out_indices  DEVICE int32 [n_heads, total_keep]: sequence-local key
 *                indices in ascending order                              -- out
 *   out_mask     DEVICE uint8 [n_heads, total_k] or NULL: 1 = selected   -- out
 * A k_b larger than the candidate count is not an argument error here: k_per_seq
 * and the candidate ranges live in device memory, which the library never reads
 * from the host, so the count is clamped on the device and the surplus index
 * slots are filled with -1 (callers that want the error check k_b on their side,
 * where they computed it).
 * -0.0 ranks equal to +0.0.
 */
pdd_status pdd_select_topk(const float *scores, int32_t n_heads, int32_t batch,
                           int32_t total_k, const int32_t *cu_seqlens_k,
                           const int32_t *cu_seqlens_k_host, int32_t max_seqlen_k,
                           const int32_t *cand_begin, const int32_t *cand_end,
                           const int32_t *k_per_seq, const int32_t *cu_keep,
                           int32_t total_keep, int32_t *out_indices, uint8_t *out_mask,
                           void *workspace, size_t workspace_bytes, pdd_stream stream);

/*
 * Selection with 1-D pooling of the scores first (Section 3.2 "Prompt Refiner":
 * after summing the weight along the query dimension, a 1-D pooling step that
 * lets neighbouring tokens be kept together, then sorting).  The paper gives neither kernel size nor type;
 * both are parameters here.  Pooled score of key j = reduction over keys
 * [j - r, j + r] of the same sequence, r = (pool_kernel - 1) / 2, stride 1:
 *   PDD_POOL_MAX  maximum over the part of the window inside the sequence
 *   PDD_POOL_AVG  sum over that part divided by pool_kernel (zero padding)
 *   PDD_POOL_NONE the raw scores (pool_kernel ignored)
 * The pooled scores are ranked exactly like pdd_select_topk ranks raw scores
 * (same arguments, same outputs).  pool_kernel must be odd, 1 .. 1025.
 *   pooled_out  DEVICE fp32 [n_heads, total_k] or NULL: the pooled scores   -- out
 */
enum { PDD_POOL_NONE = 0, PDD_POOL_MAX = 1, PDD_POOL_AVG = 2 };
pdd_status pdd_select_topk_pooled(const float *scores, int32_t n_heads, int32_t batch,
                                  int32_t total_k, const int32_t *cu_seqlens_k,
                                  const int32_t *cu_seqlens_k_host, int32_t max_seqlen_k,
                                  const int32_t *cand_begin, const int32_t *cand_end,
                                  const int32_t *k_per_seq, const int32_t *cu_keep,
                                  int32_t total_keep, int32_t pool_kernel, int32_t pool_mode,
                                  float *pooled_out, int32_t *out_indices, uint8_t *out_mask,
                                  void *workspace, size_t workspace_bytes, pdd_stream stream);

/*
 * Sentence-level selection (Section 3.2 "Prompt Refiner": the KV cache entries
 * of one sentence are combined and treated as a whole, so selecting KV cache
 * entries means selecting sentences; prefix and suffix of the prompt are not
 * refined).  Sentences are contiguous token ranges tiling the content part of
 * sequence b: sentence s (cu_sent[b] <= s < cu_sent[b+1]) covers tokens
 * [start_s, sent_end[s]) with start_s = cand_begin[b] for the first sentence and
 * sent_end[s-1] otherwise (sequence-local offsets, non-decreasing; out-of-range
 * values are clamped).  The paper does not say how token scores are combined:
 * agg_mode PDD_SENT_SUM adds them, PDD_SENT_MEAN divides the sum by the length.
 * Sentences are ranked by (score descending, index ascending) and the longest
 * prefix of the ranking whose total token count is <= token_budget[b] is kept,
 * so the refined length never exceeds the budget (k = floor(r * l), Eq. 5).
 *
 *   scores          DEVICE fp32 [n_heads, total_k]                          -- in
 *   cu_sent         DEVICE int32[B+1], sent_end DEVICE int32[total_sent]    -- in
 *   max_sent_per_seq host bound on sentences per sequence (<= 8192)
 *   cand_begin      DEVICE int32[B] or NULL (= 0)
 *   token_budget    DEVICE int32[B]
 *   out_sent_scores DEVICE fp32 [n_heads, total_sent] or NULL               -- out
 *   out_sent_keep   DEVICE uint8 [n_heads, total_sent] or NULL, 1 = kept    -- out
 *   out_mask        DEVICE uint8 [n_heads, total_k] or NULL: 1 for the tokens
 *                   of kept sentences, 0 elsewhere (also outside the content) -- out
 *   out_kept_tokens DEVICE int32 [n_heads, B] or NULL                       -- out
 */
enum { PDD_SENT_SUM = 0, PDD_SENT_MEAN = 1 };
pdd_status pdd_select_sentences(const float *scores, int32_t n_heads, int32_t batch,
                                int32_t total_k, const int32_t *cu_seqlens_k,
                                const int32_t *cu_seqlens_k_host, int32_t max_seqlen_k,
                                const int32_t *cu_sent, const int32_t *sent_end,
                                int32_t total_sent, int32_t max_sent_per_seq,
                                const int32_t *cand_begin, const int32_t *token_budget,
                                int32_t agg_mode, float *out_sent_scores,
                                uint8_t *out_sent_keep, uint8_t *out_mask,
                                int32_t *out_kept_tokens, pdd_stream stream);

/*
 * Aggregation of importance scores over attention layers and heads (Section
 * 4.4: several attention layers take part, their weight magnitudes differ, and
 * the layer strategy is left open; Section 3.2: scores are kept per head).
 * The library computes one layer per call; this entry point combines layers:
 *   out[h, j] = sum_l w_l * scores[l, h, j]              reduce_heads == 0
 *   out[0, j] = sum_l w_l * sum_h scores[l, h, j]        reduce_heads != 0
 * added to the previous contents of out when accumulate != 0 (streaming use:
 * n_layers = 1 per finished layer).  fp32, layers then heads in ascending
 * order.
 *   scores        DEVICE fp32, layer l at scores + l * layer_stride, each
 *                 [n_heads, total_k] contiguous                             -- in
 *   layer_weights DEVICE fp32[n_layers] or NULL (all 1)                     -- in
 *   out           DEVICE fp32 [reduce_heads ? 1 : n_heads, total_k]         -- out (in/out)
 */
pdd_status pdd_aggregate_scores(const float *scores, int32_t n_layers, int32_t n_heads,
                                int32_t total_k, int64_t layer_stride,
                                const float *layer_weights, int32_t reduce_heads,
                                int32_t accumulate, float *out, pdd_stream stream);

/*
 * Refinement ratio r and early-termination length L (Section 3.4 "Algorithm
 * on Refiner and Termination", program P: minimise the on-device TTFT subject
 * to Eq. 5 on r and Eq. 6 on L; Section 4.2 observes that the optimum sits at
 * L's lower bound).  Host-only scalar code, no GPU work.  With
 *   TTFT_c = k_c*l + delta_cloud                  (Eq. 2: prefill + compress + RTT)
 *   TTFT_d = TTFT_c + (delta - delta_cloud) + k_d*r*l
 *          = k_c*l + delta + k_d*r*l              (Eq. 3: + decompress + device prefill)
 * the objective grows with r, so the answer is the smallest admissible ratio:
 *   L - 1 = n = max(1, ceil((k_d*xi_scene*l - TTFT_c) / (tau - tpot_d)))   (Eq. 6, lower bound)
 *   r     = max(xi_scene, (n*tpot_c - (delta - delta_cloud)) / (k_d*l))    (Eq. 6, upper bound:
 *           a larger r lengthens the device prefill until the cloud's n tokens fit inside it)
 * provided r <= 1 - (k_c + delta/l)/k_d (Eq. 5) and k_d*r*l <= n*(tau - tpot_d) + TTFT_c.
 * Returns PDD_ERR_INFEASIBLE when no pair satisfies both constraints; *r and
 * *L are then left untouched.  Times in one unit throughout (k_* per token).
 */
typedef struct pdd_rl_model {
    double k_c, k_d;       /* prefill time per prompt token: cloud, device      */
    double delta;          /* bound on compress + decompress + RTT at length l  */
    double xi_scene;       /* smallest ratio the scenario's quality allows      */
    double tpot_c, tpot_d; /* time per output token: cloud, device              */
    double tau;            /* largest tolerable smoothed TPOT                   */
    double delta_cloud;    /* the part of delta that passes before the first
                              token reaches the device (compress + RTT);
                              0 <= delta_cloud <= delta                         */
} pdd_rl_model;
pdd_status pdd_choose_r_L(const pdd_rl_model *model, int32_t l, double *r, int32_t *L);

/*
 * Mask -> bit stream (Section 3.2: the mask tensor is treated as a bit stream
 * before compression).  For every row (head) and sequence b the stream starts
 * at a byte boundary: byte j holds tokens 8j .. 8j+7 of the sequence, first
 * token in the most significant bit, unused tail bits zero.
 *
 *   mask      DEVICE uint8 [n_rows, total_k], non-zero = selected          -- in
 *   cu_bytes  DEVICE int32[B+1] prefix sums of the per-sequence byte counts
 *             (pdd_pack_mask_layout gives ceil(Nk_b / 8) each); a count larger
 *             than that leaves the spare bytes untouched, a smaller one
 *             truncates the sequence
 *   out_bits  DEVICE uint8 [n_rows, total_bytes]                          -- out
 */
/*
 * Layout and size of that bit stream (host only, no GPU work): fills
 * cu_bytes_host[0..B] with the prefix sums of ceil(Nk_b / 8) and returns their
 * total, the number of bytes per row before compression (Section 3.2 sends the
 * compressed stream along with the first token; Section 3.2 "Prompt Refiner" and
 * Section 4.3 discuss its size).
 * Returns -1 on a NULL pointer, batch < 1 or a decreasing cu_seqlens_k_host.
 */
int64_t pdd_pack_mask_layout(int32_t batch, const int32_t *cu_seqlens_k_host, int32_t *cu_bytes_host);

pdd_status pdd_pack_mask(const uint8_t *mask, int32_t n_rows, int32_t batch, int32_t total_k,
                         const int32_t *cu_seqlens_k, const int32_t *cu_seqlens_k_host,
                         int32_t max_seqlen_k, const int32_t *cu_bytes, int32_t total_bytes,
                         uint8_t *out_bits, pdd_stream stream);

/*
 * Bytes of DEVICE scratch `which_call` can use for this descriptor (0 when it
 * has no use for any).  At most 8 * n_kv_heads * total_k * 4 bytes, for the
 * chunked call at most ceil(max_seqlen_q / 128) * n_q_heads *
 * total_k * 4 bytes and 256 MiB; never grows with Nq*Nk: the attention weights
 * are not materialised (Section 3.2 "Preliminaries").  The figure depends on
 * the descriptor, on PDD_OPT_ATTN_WAVES and on the number of compute units of
 * the current device only.  A call that is given less runs with a form that
 * needs less, or none (see pdd_prefill_attn, pdd_prefill_attn_chunked).
 */
size_t pdd_workspace_bytes(const pdd_attn_desc *desc, int which_call);

/*
 * Tuning knobs (process-wide, not thread-safe against concurrent launches).
 *   PDD_OPT_ATTN_WAVES: wavefronts per attention workgroup, 4 (128 queries) or
 *   8 (256 queries); 0 = chosen per problem (default).
 *   PDD_OPT_IMPORTANCE_KEYS: keys per workgroup of the importance kernel, 128
 *   or 256; 0 = chosen per problem (default).  Results do not depend on it.
 */
enum { PDD_OPT_ATTN_WAVES = 0, PDD_OPT_IMPORTANCE_KEYS = 1 };
pdd_status pdd_set_option(int option, int value);

/* Message for the calling thread's most recent non-OK status ("" if none). */
const char *pdd_last_error(void);

/* Library version string, e.g. "pdd 0.1 gfx950". */
const char *pdd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PDD_H */
