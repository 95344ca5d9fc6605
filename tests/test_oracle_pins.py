"""Pins for the CPU oracle: values fixed by the paper's definitions and by
mathematics, none of them produced by the oracle itself or by the GPU path."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as W
from brute import brute_packed, brute_topk

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "handworked.json")))
LN2 = float(np.log(2.0))


def bits(x):
    """float array -> bf16 bits, asserting that nothing is lost."""
    x = np.asarray(x, dtype=np.float32)
    b = W.f32_to_bf16_bits(x)
    assert np.array_equal(W.bf16_bits_to_f32(b), x), "test input must be exact in bf16"
    return b


def fr(xs):
    return np.array([float(Fraction(s)) for s in xs])


def cu(lens):
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)


# ---------------------------------------------------------------- hand-worked
def _case1_inputs():
    c = GOLD["case1"]
    q = bits(np.array(c["q"], dtype=np.float32).reshape(4, 1, 1))
    k = bits(np.array(c["k"], dtype=np.float32).reshape(4, 1, 1))
    v = bits(np.array(c["v"], dtype=np.float32).reshape(4, 1, 1))
    return q, k, v


def test_handworked_case1_attention():
    c = GOLD["case1"]
    q, k, v = _case1_inputs()
    O, lse = oracle.attention(q, k, v, cu([4]), cu([4]), LN2)
    np.testing.assert_allclose(O[:, 0, 0], fr(c["O"]), rtol=1e-13)
    np.testing.assert_allclose(np.exp(lse[0]), c["exp_LSE"], rtol=1e-13)


def test_handworked_case1_rows_of_P():
    """Row i of P is read back through V = e_j (one-hot values): O[i] = P[i,j]."""
    c = GOLD["case1"]
    q, k, _ = _case1_inputs()
    for j in range(4):
        v = np.zeros((4, 1, 1), dtype=np.float32)
        v[j] = 1.0
        O, _ = oracle.attention(q, k, bits(v), cu([4]), cu([4]), LN2)
        for i in range(4):
            want = float(Fraction(c["P_rows"][i][j])) if j <= i else 0.0
            assert abs(O[i, 0, 0] - want) < 1e-14


def test_handworked_case1_importance_and_selection():
    c = GOLD["case1"]
    q, k, _ = _case1_inputs()
    imp2 = oracle.importance(q, k, cu([4]), cu([4]), LN2, 2)
    np.testing.assert_allclose(imp2[0], fr(c["W2_imp"]), rtol=1e-13)
    imp4 = oracle.importance(q, k, cu([4]), cu([4]), LN2, 4)
    np.testing.assert_allclose(imp4[0], fr(c["W4_imp"]), rtol=1e-13)
    assert abs(imp4.sum() - 4.0) < 1e-12
    # selection on the exact fractions (ties 0 vs 2 are exact there)
    exact = fr(c["W2_imp"])[None, :]
    idx, mask = oracle.select_topk(exact, cu([4]), [2])
    assert idx[0].tolist() == c["W2_top2"] and mask[0].tolist() == [0, 1, 0, 1]
    idx, mask = oracle.select_topk(exact, cu([4]), [3])
    assert idx[0].tolist() == c["W2_top3"] and mask[0].tolist() == [1, 1, 0, 1]


def test_handworked_case2_gqa_group_sum():
    c = GOLD["case2_gqa"]
    q1, k, _ = _case1_inputs()
    q = np.zeros((4, 2, 1), dtype=np.uint16)
    q[:, 0, :] = q1[:, 0, :]                      # head A = case 1, head B = 0
    imp = oracle.importance(q, k, cu([4]), cu([4]), LN2, 2)
    np.testing.assert_allclose(imp[0], fr(c["imp_group"]), rtol=1e-13)
    assert abs(imp.sum() - c["sum"]) < 1e-12
    qB = np.zeros((4, 1, 1), dtype=np.uint16)
    impB = oracle.importance(qB, k, cu([4]), cu([4]), LN2, 2)
    np.testing.assert_allclose(impB[0], fr(c["imp_B"]), rtol=1e-13)


def test_handworked_case3_chunked():
    c = GOLD["case3_chunked"]
    q, k, v = _case1_inputs()
    qc = q[2:]
    O, lse = oracle.attention(qc, k, v, cu([2]), cu([4]), LN2)
    np.testing.assert_allclose(O[:, 0, 0], fr(c["O"]), rtol=1e-13)
    np.testing.assert_allclose(np.exp(lse[0]), c["exp_LSE"], rtol=1e-13)
    imp = oracle.importance(qc, k, cu([2]), cu([4]), LN2, -1)
    np.testing.assert_allclose(imp[0], fr(c["imp_all"]), rtol=1e-13)
    idx, mask = oracle.select_topk(fr(c["imp_all"])[None, :], cu([4]), [1],
                                   cand_begin=[0], cand_end=[2])
    assert idx[0].tolist() == c["top1_of_prefix"] and mask[0].tolist() == [0, 1, 0, 0]


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("seqs_q,seqs_k,hq,hkv,d,window,seed", [
    ([17], None, 1, 1, 8, 5, 0),
    ([33, 1, 20], None, 4, 2, 16, 7, 1),          # ragged, GQA, a length-1 prompt
    ([9, 14], None, 6, 2, 4, 64, 2),              # window longer than the prompt
    ([5, 8], [21, 8], 4, 1, 8, -1, 3),            # chunk vs prefix, all rows window
    ([6], [40], 2, 2, 32, 3, 4),                  # chunk + finite window
])
def test_oracle_matches_materialised_softmax(seqs_q, seqs_k, hq, hkv, d, window, seed):
    wl = W.make_custom("t", seqs_q, seqs_k, hq, hkv, d, max(window, 0), seed=seed)
    O, lse = oracle.attention(wl.q, wl.k, wl.v, wl.cu_seqlens_q, wl.cu_seqlens_k, wl.scale)
    imp = oracle.importance(wl.q, wl.k, wl.cu_seqlens_q, wl.cu_seqlens_k, wl.scale, window)
    bO, bL, bI = brute_packed(wl.q, wl.k, wl.v, wl.cu_seqlens_q, wl.cu_seqlens_k,
                              wl.scale, window)
    np.testing.assert_allclose(O, bO, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(lse, bL, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(imp, bI, rtol=1e-11, atol=1e-13)


def test_row_subset_equals_full_rows():
    wl = W.make_custom("t", [23, 12], None, 4, 2, 16, 4, seed=7)
    O, lse = oracle.attention(wl.q, wl.k, wl.v, wl.cu_seqlens_q, wl.cu_seqlens_k, wl.scale)
    rows = [34, 0, 22, 23, 5]
    Os, ls = oracle.attention(wl.q, wl.k, wl.v, wl.cu_seqlens_q, wl.cu_seqlens_k, wl.scale,
                              rows=rows)
    assert np.array_equal(Os, O[rows]) and np.array_equal(ls, lse[:, rows])


# ------------------------------------------------- closed forms / invariants
def _harmonic(n):
    return sum(1.0 / t for t in range(1, n + 1))


def test_uniform_case_closed_form():
    """Q = 0: every visible key gets 1/(i+delta+1); O is the running mean of V;
    LSE_i = ln(i+delta+1); importance is a difference of harmonic numbers."""
    n, hq, hkv, d, w = 40, 4, 2, 8, 12
    wl = W.make_custom("t", [n], None, hq, hkv, d, w, seed=11)
    q0 = np.zeros_like(wl.q)
    O, lse = oracle.attention(q0, wl.k, wl.v, wl.cu_seqlens_q, wl.cu_seqlens_k, wl.scale)
    v = W.bf16_bits_to_f32(wl.v).astype(np.float64)
    run_mean = np.cumsum(v, axis=0) / np.arange(1, n + 1)[:, None, None]
    for h in range(hq):
        np.testing.assert_allclose(O[:, h], run_mean[:, h // 2], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(lse[h], np.log(np.arange(1, n + 1)), rtol=1e-13, atol=1e-14)
    imp = oracle.importance(q0, wl.k, wl.cu_seqlens_q, wl.cu_seqlens_k, wl.scale, w)
    HN = _harmonic(n)
    want = np.array([(hq // hkv) * (HN - _harmonic(max(j, n - w))) for j in range(n)])
    for g in range(hkv):
        np.testing.assert_allclose(imp[g], want, rtol=1e-12)
    # an all-ties prefix: tie rule keeps the lowest indices
    idx, _ = oracle.select_topk(imp, wl.cu_seqlens_k, [10])
    assert idx[0].tolist() == list(range(10))


def test_row0_and_single_token_prompts_give_the_dot_product():
    """A prompt of one token: P = [1], O = v, LSE = scale * <q, k>  (checks the
    contraction against numpy's matmul on the widened inputs)."""
    b, hq, hkv, d = 12, 4, 2, 32
    wl = W.make_custom("t", [1] * b, None, hq, hkv, d, 1, seed=5)
    O, lse = oracle.attention(wl.q, wl.k, wl.v, wl.cu_seqlens_q, wl.cu_seqlens_k, 0.37)
    q = W.bf16_bits_to_f32(wl.q).astype(np.float64)
    k = W.bf16_bits_to_f32(wl.k).astype(np.float64)
    v = W.bf16_bits_to_f32(wl.v).astype(np.float64)
    for h in range(hq):
        want = 0.37 * np.einsum("bc,bc->b", q[:, h], k[:, h // 2])
        np.testing.assert_allclose(lse[h], want, rtol=1e-13, atol=1e-14)
        np.testing.assert_array_equal(O[:, h], v[:, h // 2])
    imp = oracle.importance(wl.q, wl.k, wl.cu_seqlens_q, wl.cu_seqlens_k, 0.37, 1)
    np.testing.assert_allclose(imp, (hq // hkv) * np.ones_like(imp), rtol=1e-13)


def test_rows_sum_to_one_and_importance_mass():
    """V = 1 reads back the row sums; sum_j imp[g,j] = G * W_b per sequence."""
    lens, hq, hkv, d, w = [30, 7, 19], 6, 3, 16, 10
    wl = W.make_custom("t", lens, None, hq, hkv, d, w, seed=9)
    ones = bits(np.ones(wl.v.shape, dtype=np.float32))
    O, _ = oracle.attention(wl.q, wl.k, ones, wl.cu_seqlens_q, wl.cu_seqlens_k, wl.scale)
    np.testing.assert_allclose(O, 1.0, rtol=0, atol=1e-12)
    imp = oracle.importance(wl.q, wl.k, wl.cu_seqlens_q, wl.cu_seqlens_k, wl.scale, w)
    assert (imp >= 0).all()
    for b, n in enumerate(lens):
        seg = imp[:, wl.cu_seqlens_k[b]:wl.cu_seqlens_k[b + 1]]
        np.testing.assert_allclose(seg.sum(axis=1), (hq // hkv) * min(w, n), rtol=1e-12)
    # W = N: the column sums of one head total N
    wl1 = W.make_custom("t", [25], None, 1, 1, 8, 25, seed=10)
    imp1 = oracle.importance(wl1.q, wl1.k, wl1.cu_seqlens_q, wl1.cu_seqlens_k, wl1.scale, 25)
    assert abs(imp1.sum() - 25.0) < 1e-11


def test_causal_mask_bounds_on_importance():
    """Key j only receives mass from window queries i with i + delta >= j; the
    last key is seen by the last query alone."""
    n, hq, hkv, d, w = 24, 2, 1, 8, 6
    wl = W.make_custom("t", [n], None, hq, hkv, d, w, seed=13)
    imp = oracle.importance(wl.q, wl.k, wl.cu_seqlens_q, wl.cu_seqlens_k, wl.scale, w)
    for j in range(n):
        n_seen_by = n - max(j, n - w)
        assert imp[0, j] <= hq * n_seen_by + 1e-12
    # read P[n-1, n-1] of each head through a one-hot V
    v = np.zeros((n, 1, d), dtype=np.float32)
    v[n - 1, 0, 0] = 1.0
    O, _ = oracle.attention(wl.q, wl.k, bits(v), wl.cu_seqlens_q, wl.cu_seqlens_k, wl.scale,
                            rows=[n - 1])
    assert abs(imp[0, n - 1] - O[0, :, 0].sum()) < 1e-14
    # a strictly later key than every window query is impossible here, but a
    # chunk never attends past its own position: with delta = 3 the key at
    # local index nq-1+delta+... does not exist; check delta handling instead
    wlc = W.make_custom("t", [4], [9], 1, 1, 8, 0, seed=14, chunked=True)
    impc = oracle.importance(wlc.q, wlc.k, wlc.cu_seqlens_q, wlc.cu_seqlens_k, wlc.scale, -1)
    assert abs(impc.sum() - 4.0) < 1e-12
    # the last three keys are seen by 3, 2, 1 chunk queries only
    assert impc[0, 8] <= 1 and impc[0, 7] <= 2 and impc[0, 6] <= 3


def test_key_shift_leaves_P_unchanged_and_moves_lse():
    """k_j <- k_j + c for all j: P and O do not change, LSE_i grows by
    scale * <q_i, c> (integers keep everything exact in bf16); a large shift
    also exercises the max subtraction."""
    rng = np.random.default_rng(21)
    n, d = 20, 4
    q = rng.integers(-2, 3, size=(n, 1, d)).astype(np.float32)
    k = rng.integers(-3, 4, size=(n, 1, d)).astype(np.float32)
    v = rng.integers(-8, 9, size=(n, 1, d)).astype(np.float32)
    c = np.array([40, -24, 16, 56], dtype=np.float32)
    O1, l1 = oracle.attention(bits(q), bits(k), bits(v), cu([n]), cu([n]), 0.5)
    O2, l2 = oracle.attention(bits(q), bits(k + c), bits(v), cu([n]), cu([n]), 0.5)
    np.testing.assert_allclose(O1, O2, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(l2[0] - l1[0], 0.5 * (q[:, 0, :] @ c), rtol=1e-11, atol=1e-11)
    i1 = oracle.importance(bits(q), bits(k), cu([n]), cu([n]), 0.5, 5)
    i2 = oracle.importance(bits(q), bits(k + c), cu([n]), cu([n]), 0.5, 5)
    np.testing.assert_allclose(i1, i2, rtol=1e-10, atol=1e-13)


def test_identities_chunked_ragged_gqa():
    hq, hkv, d = 4, 2, 16
    full = W.make_custom("t", [37], None, hq, hkv, d, 9, seed=17)
    O, lse = oracle.attention(full.q, full.k, full.v, cu([37]), cu([37]), full.scale)
    imp = oracle.importance(full.q, full.k, cu([37]), cu([37]), full.scale, 9)
    # chunked(Q[P:]) == rows [P, N) of the full run, importance == W = chunk
    P = 28
    Oc, lc = oracle.attention(full.q[P:], full.k, full.v, cu([9]), cu([37]), full.scale)
    ic = oracle.importance(full.q[P:], full.k, cu([9]), cu([37]), full.scale, -1)
    assert np.array_equal(Oc, O[P:]) and np.array_equal(lc, lse[:, P:])
    np.testing.assert_allclose(ic, imp, rtol=1e-14)
    # packed == alone
    two = W.make_custom("t", [11, 26], None, hq, hkv, d, 5, seed=18)
    Ot, lt = oracle.attention(two.q, two.k, two.v, two.cu_seqlens_q, two.cu_seqlens_k, two.scale)
    it = oracle.importance(two.q, two.k, two.cu_seqlens_q, two.cu_seqlens_k, two.scale, 5)
    Oa, la = oracle.attention(two.q[11:], two.k[11:], two.v[11:], cu([26]), cu([26]), two.scale)
    ia = oracle.importance(two.q[11:], two.k[11:], cu([26]), cu([26]), two.scale, 5)
    assert np.array_equal(Ot[11:], Oa) and np.array_equal(lt[:, 11:], la)
    assert np.array_equal(it[:, 11:], ia)
    # GQA == MHA with repeated K,V ; group importance = sum over repeated heads
    kr = np.repeat(full.k, hq // hkv, axis=1)
    vr = np.repeat(full.v, hq // hkv, axis=1)
    Om, lm = oracle.attention(full.q, kr, vr, cu([37]), cu([37]), full.scale)
    im = oracle.importance(full.q, kr, cu([37]), cu([37]), full.scale, 9)
    assert np.array_equal(Om, O) and np.array_equal(lm, lse)
    np.testing.assert_allclose(im.reshape(hkv, hq // hkv, -1).sum(axis=1), imp, rtol=1e-13)


# ---------------------------------------------------------------- selection
def test_select_matches_rank_counting_with_ties():
    rng = np.random.default_rng(3)
    lens = [13, 1, 30]
    scores = rng.integers(0, 6, size=(2, sum(lens))).astype(np.float64) / 4.0  # many ties
    ks = [5, 1, 11]
    idx, mask = oracle.select_topk(scores, cu(lens), ks)
    cuk = cu(lens)
    cukeep = np.concatenate([[0], np.cumsum(ks)])
    for g in range(2):
        for b in range(3):
            row = scores[g, cuk[b]:cuk[b + 1]]
            want = brute_topk(row, ks[b])
            got = idx[g, cukeep[b]:cukeep[b + 1]]
            assert got.tolist() == want.tolist()
            assert (np.diff(got) > 0).all() if len(got) > 1 else True
            m = mask[g, cuk[b]:cuk[b + 1]]
            assert m.sum() == ks[b] and set(np.nonzero(m)[0]) == set(got)
            if ks[b] < len(row):
                assert row[got].min() >= np.delete(row, got).max()


def test_select_candidate_range_and_edge_counts():
    s = np.array([[9.0, 1.0, 5.0, 7.0, 3.0, 8.0]])
    idx, mask = oracle.select_topk(s, cu([6]), [2], cand_begin=[1], cand_end=[5])
    assert idx[0].tolist() == [2, 3] and mask[0].tolist() == [0, 0, 1, 1, 0, 0]
    idx, mask = oracle.select_topk(s, cu([6]), [0])
    assert idx.shape == (1, 0) and mask.sum() == 0
    idx, mask = oracle.select_topk(s, cu([6]), [6])
    assert idx[0].tolist() == [0, 1, 2, 3, 4, 5]
    with pytest.raises(ValueError):
        oracle.select_topk(s, cu([6]), [5], cand_begin=[1], cand_end=[5])


# ---------------------------------------------------------------- workloads
def test_workload_recipes():
    assert W.c3_lengths_from_recipe() == W.C3_LENGTHS
    assert [W.keep_count(n, r) for n, r in
            [(512, "1/2"), (4096, "3/10"), (32768, "1/10"), (8192, "1/4"), (3, "1/10")]] == \
        [256, 1228, 3276, 2048, 1]
    c1 = W.make_workload("c1")
    assert c1.causal_pairs() == 131328 and c1.window_pairs() == 15888
    c5 = W.make_workload("c5", n_override=64)
    assert c5.cand_end.tolist() == [64] * 4 and c5.seqlens_k.tolist() == [320] * 4
    x = np.array([1.0, 1.00390625, 1.01171875, -3.5e-41], dtype=np.float32)
    assert W.f32_to_bf16_bits(x).tolist()[:3] == [0x3F80, 0x3F80, 0x3F82]


# ---------------------------------------------------------------- bit stream
def test_pack_mask_hand_example_and_roundtrip():
    """Tokens [1,0,0,0,0,0,0,1 | 1,1] then [0,1,0]: first token in the most
    significant bit, each sequence byte aligned -> 0b10000001, 0b11000000, 0b01000000."""
    bits, cu_bytes = oracle.pack_mask(np.array([[1, 0, 0, 0, 0, 0, 0, 1, 1, 1, 0, 1, 0]]), [0, 10, 13])
    assert bits.tolist() == [[0x81, 0xC0, 0x40]] and cu_bytes.tolist() == [0, 2, 3]
    rng = np.random.default_rng(4)
    lens = [5, 16, 0, 37]
    m = rng.integers(0, 2, size=(3, sum(lens))).astype(np.uint8)
    bits, cb = oracle.pack_mask(m * 7, cu(lens))          # any non-zero byte counts as selected
    cuk = cu(lens)
    for r in range(3):
        for b, n in enumerate(lens):
            got = [(bits[r, cb[b] + j // 8] >> (7 - j % 8)) & 1 for j in range(n)]
            assert got == m[r, cuk[b]:cuk[b + 1]].tolist()
            tail = bits[r, cb[b]:cb[b + 1]]
            if n % 8:
                assert tail[-1] & ((1 << (8 - n % 8)) - 1) == 0     # unused tail bits are zero


# ---------------------------------------------------------------- 1-D pooling
def test_pool_scores_hand_example_and_library_special_case():
    s = np.array([[1.0, 5.0, 2.0, 0.0, 4.0, 3.0, 9.0]])
    got = oracle.pool_scores(s, [0, 4, 7], 3, "max")        # two sequences: [1,5,2,0] and [4,3,9]
    assert got.tolist() == [[5.0, 5.0, 5.0, 2.0, 4.0, 9.0, 9.0]]
    got = oracle.pool_scores(s, [0, 4, 7], 3, "avg")        # zero padding, divide by 3
    np.testing.assert_allclose(got, [[2.0, 8 / 3, 7 / 3, 2 / 3, 7 / 3, 16 / 3, 4.0]], rtol=1e-15)
    assert np.array_equal(oracle.pool_scores(s, [0, 4, 7], 1, "avg"), s)
    # one sequence: equals the library's pooling with padding k//2, stride 1
    import torch
    import torch.nn.functional as F
    x = np.random.default_rng(0).random((3, 50))
    for k in (3, 5, 9):
        t = torch.from_numpy(x)[None]
        np.testing.assert_allclose(oracle.pool_scores(x, [0, 50], k, "max"),
                                   F.max_pool1d(t, k, stride=1, padding=k // 2)[0].numpy(), rtol=0)
        np.testing.assert_allclose(oracle.pool_scores(x, [0, 50], k, "avg"),
                                   F.avg_pool1d(t, k, stride=1, padding=k // 2)[0].numpy(), rtol=1e-14)


# ------------------------------------------------- sentence-level selection
def test_select_sentences_hand_example():
    # one sequence of 12 tokens, content [2, 11): sentences [2,5) [5,6) [6,10) [10,11)
    s = np.array([[9, 9, 1, 2, 3, 8, 1, 1, 1, 1, 5, 9]], dtype=np.float64)
    ends = [5, 6, 10, 11]
    # sums 6, 8, 4, 5 -> ranking 1, 0, 3, 2 with lengths 1, 3, 1, 4
    sc, keep, mask, kept = oracle.select_sentences(s, [0, 12], [0, 4], ends, [5], "sum", [2])
    assert sc.tolist() == [[6, 8, 4, 5]]
    assert keep.tolist() == [[1, 1, 0, 1]] and kept.tolist() == [[5]]
    assert mask.tolist() == [[0, 0, 1, 1, 1, 1, 0, 0, 0, 0, 1, 0]]
    # budget 4: after sentences 1 and 0 the next one in the ranking (3, length 1) would make 5 > 4:
    # the kept set is a PREFIX of the ranking, nothing further down is tried
    _, keep, _, kept = oracle.select_sentences(s, [0, 12], [0, 4], ends, [4], "sum", [2])
    assert keep.tolist() == [[1, 1, 0, 0]] and kept.tolist() == [[4]]
    # budget 3: sentence 1 (len 1) fits, sentence 0 (len 3) does not -> stop
    _, keep, _, kept = oracle.select_sentences(s, [0, 12], [0, 4], ends, [3], "sum", [2])
    assert keep.tolist() == [[0, 1, 0, 0]] and kept.tolist() == [[1]]
    # means 2, 8, 1, 5 -> ranking 1, 3, 0, 2; budget 5 keeps all but the longest
    sc, keep, mask, kept = oracle.select_sentences(s, [0, 12], [0, 4], ends, [5], "mean", [2])
    assert sc.tolist() == [[2, 8, 1, 5]]
    assert keep.tolist() == [[1, 1, 0, 1]] and kept.tolist() == [[5]]
    # budget 2 under means: ranking 1 (len 1), 3 (len 1), then 0 (len 3) stops
    _, keep, mask, kept = oracle.select_sentences(s, [0, 12], [0, 4], ends, [2], "mean", [2])
    assert keep.tolist() == [[0, 1, 0, 1]] and kept.tolist() == [[2]]
    assert mask.tolist() == [[0, 0, 0, 0, 0, 1, 0, 0, 0, 0, 1, 0]]
    # ties go to the earlier sentence
    t = np.array([[1, 1, 1, 1]], dtype=np.float64)
    _, keep, _, _ = oracle.select_sentences(t, [0, 4], [0, 4], [1, 2, 3, 4], [2], "sum")
    assert keep.tolist() == [[1, 1, 0, 0]]


def test_select_sentences_reduces_to_token_topk_and_invariants():
    rng = np.random.default_rng(21)
    lens = [57, 1, 200]
    cu = np.concatenate([[0], np.cumsum(lens)])
    s = rng.random((3, sum(lens)))
    s[1, 60:90] = 0.25                                   # ties
    cb = np.array([3, 0, 10]); ce = np.array([50, 1, 190]); kk = np.array([11, 1, 60])
    # every token its own sentence: the rule becomes plain top-k over the candidate range
    ends = np.concatenate([np.arange(cb[b] + 1, ce[b] + 1) for b in range(3)])
    cu_sent = np.concatenate([[0], np.cumsum(ce - cb)])
    for mode in ("sum", "mean"):
        _, keep, mask, kept = oracle.select_sentences(s, cu, cu_sent, ends, kk, mode, cb)
        idx, mask_tok = oracle.select_topk(s, cu, kk, cb, ce)
        assert np.array_equal(mask, mask_tok)
        assert np.array_equal(kept, np.tile(kk, (3, 1)))
    # random sentence splits: the kept set is the longest ranking prefix that fits
    for seed in range(5):
        r = np.random.default_rng(seed)
        n = 250
        cuts = np.sort(r.choice(np.arange(11, 240), size=25, replace=False))
        ends = np.concatenate([cuts, [240]])
        sc, keep, mask, kept = oracle.select_sentences(s[:1, :n], [0, n], [0, 26], ends, [120], "mean", [10])
        starts = np.concatenate([[10], ends[:-1]])
        ln = ends - starts
        np.testing.assert_allclose(sc[0], [s[0, a:b].mean() for a, b in zip(starts, ends)], rtol=1e-13)
        assert kept[0, 0] == ln[keep[0] == 1].sum() == mask.sum() <= 120
        assert mask[0, :10].sum() == 0 and mask[0, 240:].sum() == 0
        for a, b, f in zip(starts, ends, keep[0]):
            assert (mask[0, a:b] == f).all()
        # every kept sentence outranks every dropped one, and the best dropped one does not fit
        if (keep[0] == 0).any() and (keep[0] == 1).any():
            assert sc[0][keep[0] == 1].min() >= sc[0][keep[0] == 0].max()
        if (keep[0] == 0).any():
            best_dropped = np.flatnonzero(keep[0] == 0)[np.argmax(sc[0][keep[0] == 0])]
            assert kept[0, 0] + ln[best_dropped] > 120


# ------------------------------------- cross-layer aggregation, (r, L) chooser
def test_aggregate_scores_pins():
    s = np.arange(2 * 3 * 4, dtype=np.float64).reshape(2, 3, 4)
    # hand values: layer 0 rows 0..11, layer 1 rows 12..23
    got = oracle.aggregate_scores(s, [1.0, 0.5])
    assert got.tolist() == [[6, 7.5, 9, 10.5], [12, 13.5, 15, 16.5], [18, 19.5, 21, 22.5]]
    got = oracle.aggregate_scores(s, [1.0, 0.5], reduce_heads=True)
    assert got.tolist() == [[36, 40.5, 45, 49.5]]
    rng = np.random.default_rng(0)
    x = rng.random((5, 4, 33)); w = rng.random(5)
    np.testing.assert_allclose(oracle.aggregate_scores(x, w), np.einsum("l,lhn->hn", w, x), rtol=1e-14)
    np.testing.assert_allclose(oracle.aggregate_scores(x, None, True), x.sum((0, 1))[None], rtol=1e-14)
    one_hot = np.zeros(5); one_hot[3] = 1
    assert np.array_equal(oracle.aggregate_scores(x, one_hot), x[3])
    acc = rng.random((4, 33))
    np.testing.assert_allclose(oracle.aggregate_scores(x, w, acc=acc), acc + np.einsum("l,lhn->hn", w, x), rtol=1e-14)


def test_choose_r_L_search_matches_closed_form():
    # the objective grows with r, so r* = xi_scene whenever Eq. 5 leaves room; L* = the smallest
    # integer >= 2 meeting the smoothed-TPOT bound, valid only below the cloud-occupation bound
    import math
    cases = [dict(l=8192, k_c=0.02, k_d=0.5, delta=300, xi_scene=0.6, tpot_c=30, tpot_d=50, tau=100),
             dict(l=4096, k_c=0.05, k_d=0.4, delta=150, xi_scene=0.25, tpot_c=20, tpot_d=40, tau=100),
             dict(l=32768, k_c=0.01, k_d=0.3, delta=500, xi_scene=0.5, tpot_c=25, tpot_d=60, tau=120),
             dict(l=100, k_c=0.3, k_d=0.5, delta=5, xi_scene=0.2, tpot_c=10, tpot_d=50, tau=100)]
    for c in cases:
        got = oracle.choose_r_L(**c)
        lo = (c["k_d"] * c["xi_scene"] * c["l"] - c["k_c"] * c["l"]) / (c["tau"] - c["tpot_d"])
        assert got is not None
        assert got[0] == c["xi_scene"] and got[1] == 1 + max(1, math.ceil(lo))
    # worked numbers for the first case: prefill_d = 2457.6, TTFT_c = 163.84 -> (2293.76 / 50) = 45.9 -> L = 47
    assert oracle.choose_r_L(**cases[0]) == (0.6, 47)
    # the part of delta spent before the first token arrives (compress + RTT, Eq. 2) delays TTFT_c:
    # TTFT_c = 163.84 + 200 -> (2457.6 - 363.84) / 50 = 41.875 -> L = 43; the cloud-occupation bound
    # is (decompress + prefill_d) / TPOT_c = (100 + 2457.6) / 30 = 85.25 (Eq. 3, Eq. 6)
    assert oracle.choose_r_L(**cases[0], delta_cloud=200) == (0.6, 43)
    # a case the split decides: prefill_d(rl) = 10, lower bound <= 0 -> L - 1 = 1; the upper bound is
    # (5 - delta_cloud + 10) / 12: 1.25 with delta_cloud = 0 (feasible, L = 2), 0.83 with delta_cloud = 5
    tight = dict(l=100, k_c=0.3, k_d=0.5, delta=5, xi_scene=0.2, tpot_c=12, tpot_d=50, tau=100)
    assert oracle.choose_r_L(**tight) == (0.2, 2)
    # with delta_cloud = 5 the ratio xi_scene = 0.2 is infeasible, but P is not: the bound 0.5 r 100 / 12 >= 1
    # holds from r = 0.24 on (Eq. 5 allows r <= 1 - (0.3 + 0.05) / 0.5 = 0.3), so the optimum moves there
    assert oracle.choose_r_L(**tight, delta_cloud=5) == (0.24, 2)
    assert oracle.choose_r_L(**dict(tight, tpot_c=16), delta_cloud=5) is None       # would need r = 0.32 > 0.3
    # off-grid optimum: tpot_c = 12.3 -> r = 12.3 / 50 = 0.246
    assert oracle.choose_r_L(**dict(tight, tpot_c=12.3), delta_cloud=5) == (float(__import__("fractions").Fraction(12.3) / 50), 2)
    # Eq. 5 empty: the cloud is too slow relative to the device
    assert oracle.choose_r_L(8192, 0.4, 0.5, 300, 0.6, 30, 50, 100) is None
    # Eq. 6 empty: the smoothing needs more cloud tokens than the occupation bound allows
    assert oracle.choose_r_L(8192, 0.02, 0.5, 300, 0.6, 300, 50, 60) is None


# --------------------------------------- hand-worked fixture of the refinement stages
def test_refinement_stages_against_the_hand_worked_fixture():
    """tests/golden/refinement_handworked.json: sentence-level selection, pooling, bit stream
    and layer aggregation worked by hand from the definitions."""
    import json
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "refinement_handworked.json")) as f:
        fx = json.load(f)
    s = fx["sentences"]
    sc = np.array([s["scores"]], dtype=np.float64)
    n, ends, cb = len(s["scores"]), s["sentence_ends"], [s["content_begin"]]
    run = lambda mode, budget: oracle.select_sentences(sc, [0, n], [0, len(ends)], ends, [budget], mode, cb)
    assert run("sum", 5)[0].tolist() == [s["sums"]] and run("mean", 5)[0].tolist() == [s["means"]]
    assert run("sum", 5)[1].tolist() == [s["sum_budget5_keep"]] and run("sum", 5)[2].tolist() == [s["sum_budget5_mask"]]
    assert run("sum", 4)[1].tolist() == [s["sum_budget4_keep"]]
    assert run("sum", 3)[1].tolist() == [s["sum_budget3_keep"]]
    assert run("mean", 5)[1].tolist() == [s["mean_budget5_keep"]]
    assert run("mean", 2)[1].tolist() == [s["mean_budget2_keep"]] and run("mean", 2)[2].tolist() == [s["mean_budget2_mask"]]
    p = fx["pooling"]
    ps = np.array([p["scores"]], dtype=np.float64)
    assert oracle.pool_scores(ps, p["cu_seqlens"], 3, "max").tolist() == [p["max_k3"]]
    np.testing.assert_allclose(3 * oracle.pool_scores(ps, p["cu_seqlens"], 3, "avg"), [p["avg_k3_times3"]], rtol=1e-15)
    b = fx["bit_stream"]
    bits, _ = oracle.pack_mask(np.array([b["mask"]], dtype=np.uint8), b["cu_seqlens"])
    assert bits.tolist() == [b["bytes"]]
    a = fx["aggregation"]
    stack = np.arange(24, dtype=np.float64).reshape(2, 3, 4)
    assert oracle.aggregate_scores(stack, a["weights"]).tolist() == a["per_head"]
    assert oracle.aggregate_scores(stack, a["weights"], reduce_heads=True).tolist() == a["heads_reduced"]
