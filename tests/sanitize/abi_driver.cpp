// Host-only driver for the sanitizer pass over the C ABI's validation layer: every call here
// is rejected (or answered) on the host before anything could be launched, so it runs without a
// GPU.  Built with AddressSanitizer and UndefinedBehaviorSanitizer on the host code of
// pdd_api.hip; a sanitizer report makes the process exit non-zero.
#include "../../include/pdd.h"
#include <cstdio>
#include <cstring>
#include <vector>

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED: %s (line %d): %s\n", #cond, __LINE__, pdd_last_error()); ++failures; } } while (0)

static pdd_attn_desc good_desc()
{
    pdd_attn_desc d;
    std::memset(&d, 0, sizeof d);
    d.batch = 1; d.n_q_heads = 4; d.n_kv_heads = 2; d.head_dim = 128;
    d.total_q = d.total_k = d.max_seqlen_q = d.max_seqlen_k = 64;
    d.cu_seqlens_q = d.cu_seqlens_k = reinterpret_cast<const int32_t *>(0x1000);   // never followed
    d.q_stride_tok = d.o_stride_tok = 4 * 128; d.k_stride_tok = d.v_stride_tok = 2 * 128;
    d.q_stride_head = d.k_stride_head = d.v_stride_head = d.o_stride_head = 128;
    d.window = 8;
    return d;
}

int main()
{
    void *const q = (void *)0x10000, *const k = (void *)0x20000, *const v = (void *)0x30000, *const o = (void *)0x40000;
    float *const lse = (float *)0x50000, *const imp = (float *)0x60000;
    pdd_attn_desc d = good_desc();
    EXPECT(pdd_prefill_attn(nullptr, q, k, v, o, lse, imp, nullptr, 0, nullptr) == PDD_ERR_INVALID_ARG);
    d.n_kv_heads = 3;   EXPECT(pdd_prefill_attn(&d, q, k, v, o, lse, imp, nullptr, 0, nullptr) == PDD_ERR_INVALID_ARG);
    d = good_desc(); d.head_dim = 96;   EXPECT(pdd_prefill_attn(&d, q, k, v, o, lse, imp, nullptr, 0, nullptr) == PDD_ERR_UNSUPPORTED);
    d = good_desc(); d.q_stride_tok = 100;   EXPECT(pdd_prefill_attn(&d, q, k, v, o, lse, imp, nullptr, 0, nullptr) == PDD_ERR_INVALID_ARG);
    d = good_desc();   EXPECT(pdd_prefill_attn(&d, q, k, (void *)0x30008, o, lse, imp, nullptr, 0, nullptr) == PDD_ERR_INVALID_ARG);
    EXPECT(pdd_prefill_attn(&d, q, k, v, o, lse, nullptr, nullptr, 0, nullptr) == PDD_ERR_INVALID_ARG);
    // host copies of cu_seqlens: every rejection path reads the arrays
    {
        const int32_t bad0[2] = {1, 64}, bad1[2] = {0, 63}, bad2[2] = {0, 70};
        d = good_desc(); d.cu_seqlens_q_host = bad0;   EXPECT(pdd_prefill_attn(&d, q, k, v, o, lse, imp, nullptr, 0, nullptr) == PDD_ERR_INVALID_ARG);
        d.cu_seqlens_q_host = bad1;   EXPECT(pdd_prefill_attn(&d, q, k, v, o, lse, imp, nullptr, 0, nullptr) == PDD_ERR_INVALID_ARG);
        d.cu_seqlens_q_host = bad2;   EXPECT(pdd_prefill_attn(&d, q, k, v, o, lse, imp, nullptr, 0, nullptr) == PDD_ERR_INVALID_ARG);
        const int32_t cq[3] = {0, 40, 64}, ck[3] = {0, 30, 80};
        d = good_desc(); d.batch = 2; d.total_k = 80; d.max_seqlen_k = 60; d.cu_seqlens_q_host = cq; d.cu_seqlens_k_host = ck;
        EXPECT(pdd_prefill_attn_chunked(&d, q, k, v, o, lse, imp, nullptr, 0, nullptr) == PDD_ERR_INVALID_ARG);
        EXPECT(pdd_prefill_attn_chunked_noalloc(&d, q, k, v, o, lse, imp, nullptr) == PDD_ERR_INVALID_ARG);
    }
    d = good_desc(); d.window = 0;   EXPECT(pdd_token_importance(&d, q, k, lse, imp, nullptr, 0, nullptr) == PDD_ERR_INVALID_ARG);
    // scratch sizes
    d = good_desc();   EXPECT(pdd_workspace_bytes(&d, PDD_CALL_PREFILL_ATTN) == 0);
    d.batch = 4; d.n_q_heads = 64; d.n_kv_heads = 8; d.total_q = 1024; d.max_seqlen_q = 256; d.total_k = 4 * 8448; d.max_seqlen_k = 8448;
    EXPECT(pdd_workspace_bytes(&d, PDD_CALL_PREFILL_ATTN_CHUNKED) % ((size_t)8 * 4 * 8448 * 4) == 0);
    EXPECT(pdd_workspace_bytes(nullptr, 0) == 0);
    // selection family
    const float *sc = (const float *)0x1000;  const int32_t *dev = (const int32_t *)0x2000;  int32_t *idx = (int32_t *)0x3000;
    EXPECT(pdd_select_topk(nullptr, 2, 1, 64, dev, nullptr, 64, nullptr, nullptr, dev, dev, 8, idx, nullptr, nullptr, 0, nullptr) == PDD_ERR_INVALID_ARG);
    EXPECT(pdd_select_topk(sc, 2, 1, 64, dev, nullptr, 65, nullptr, nullptr, dev, dev, 8, idx, nullptr, nullptr, 0, nullptr) == PDD_ERR_INVALID_ARG);
    EXPECT(pdd_select_topk(sc, 2, 1, 64, dev, nullptr, 64, dev, nullptr, dev, dev, 8, idx, nullptr, nullptr, 0, nullptr) == PDD_ERR_INVALID_ARG);
    EXPECT(pdd_select_topk_pooled(sc, 2, 1, 64, dev, nullptr, 64, nullptr, nullptr, dev, dev, 8, 4, PDD_POOL_MAX, nullptr, idx, nullptr, nullptr, 0, nullptr) == PDD_ERR_INVALID_ARG);
    EXPECT(pdd_select_sentences(sc, 2, 1, 64, dev, nullptr, 64, dev, dev, 20000, 9000, nullptr, dev, PDD_SENT_SUM, nullptr, nullptr, nullptr, nullptr, nullptr) == PDD_ERR_UNSUPPORTED);
    EXPECT(pdd_pack_mask(nullptr, 2, 1, 64, dev, nullptr, 64, dev, 8, (uint8_t *)0x4000, nullptr) == PDD_ERR_INVALID_ARG);
    EXPECT(pdd_aggregate_scores(sc, 2, 8, 64, 100, nullptr, 0, 0, (float *)0x5000, nullptr) == PDD_ERR_INVALID_ARG);
    // host-only helpers
    {
        const int32_t cu[4] = {0, 13, 13, 77};
        int32_t cu_bytes[4];
        EXPECT(pdd_pack_mask_layout(3, cu, cu_bytes) == 2 + 0 + 8 && cu_bytes[3] == 10);
        const int32_t dec[3] = {0, 5, 3};
        EXPECT(pdd_pack_mask_layout(2, dec, cu_bytes) == -1);
        pdd_rl_model m = {0.02, 0.5, 300, 0.6, 30, 50, 100, 200};
        double r = 0; int32_t L = 0;
        EXPECT(pdd_choose_r_L(&m, 8192, &r, &L) == PDD_OK && L == 43 && r == 0.6);
        m.tpot_c = 300; m.tau = 60;
        EXPECT(pdd_choose_r_L(&m, 8192, &r, &L) == PDD_ERR_INFEASIBLE);
        EXPECT(pdd_choose_r_L(&m, 0, &r, &L) == PDD_ERR_INVALID_ARG);
    }
    EXPECT(pdd_set_option(99, 1) == PDD_ERR_INVALID_ARG);
    EXPECT(std::strlen(pdd_version()) > 0);
    std::printf(failures ? "abi driver: %d check(s) failed\n" : "abi driver: all checks passed\n", failures);
    return failures ? 1 : 0;
}
