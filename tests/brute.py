"""Independent second statement of the method for tiny inputs (N <= ~100).

Materialises the full masked softmax(Q K^T * s) matrix with numpy matmuls and
normalises by division -- a different formulation from the oracle's per-row
exp(S - LSE) loops -- so that an indexing, sign or transposition mistake in
the oracle shows up as a disagreement.  (Section 2.2.3 attention equation;
Section 3.2 "Prompt Refiner".)
"""
import numpy as np


def widen(bits):
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def brute_sequence(q, k, v, scale, window):
    """q [Nq,Hq,d], k/v [Nk,Hkv,d] float64 for ONE sequence.
    Returns P [Hq,Nq,Nk], O [Nq,Hq,d], LSE [Hq,Nq], imp [Hkv,Nk]."""
    nq, hq, d = q.shape
    nk, hkv, _ = k.shape
    grp = hq // hkv
    delta = nk - nq
    ii = np.arange(nq)[:, None]
    jj = np.arange(nk)[None, :]
    visible = jj <= ii + delta
    P = np.zeros((hq, nq, nk))
    O = np.zeros((nq, hq, d))
    LSE = np.zeros((hq, nq))
    imp = np.zeros((hkv, nk))
    w = nq if window < 0 else min(window, nq)
    for h in range(hq):
        g = h // grp
        S = (q[:, h, :] @ k[:, g, :].T) * scale
        S = np.where(visible, S, -np.inf)
        E = np.exp(S - S.max(axis=1, keepdims=True))
        Z = E.sum(axis=1, keepdims=True)
        P[h] = E / Z
        O[:, h, :] = P[h] @ v[:, g, :]
        LSE[h] = np.log(Z[:, 0]) + S.max(axis=1)
        if w > 0:
            imp[g] += P[h][nq - w:, :].sum(axis=0)
    return P, O, LSE, imp


def brute_packed(wl_q, wl_k, wl_v, cu_q, cu_k, scale, window):
    """Packed batch of bf16 bit patterns -> O [total_q,Hq,d], LSE [Hq,total_q],
    imp [Hkv,total_k] by running `brute_sequence` on each sequence alone."""
    q, k, v = widen(wl_q), widen(wl_k), widen(wl_v)
    tq, hq, d = q.shape
    tk, hkv, _ = k.shape
    O = np.zeros((tq, hq, d))
    LSE = np.zeros((hq, tq))
    imp = np.zeros((hkv, tk))
    for b in range(len(cu_q) - 1):
        qs, qe, ks, ke = cu_q[b], cu_q[b + 1], cu_k[b], cu_k[b + 1]
        if qe == qs:
            continue
        _, o, l, im = brute_sequence(q[qs:qe], k[ks:ke], v[ks:ke], scale, window)
        O[qs:qe] = o
        LSE[:, qs:qe] = l
        imp[:, ks:ke] = im
    return O, LSE, imp


def brute_topk(scores_row, k):
    """Rank by counting: index j is kept iff fewer than k candidates beat it,
    where a beats j when score[a] > score[j], or equal and a < j."""
    s = np.asarray(scores_row, dtype=np.float64)
    n = len(s)
    keep = []
    for j in range(n):
        beats = 0
        for a in range(n):
            if s[a] > s[j] or (s[a] == s[j] and a < j):
                beats += 1
        if beats < k:
            keep.append(j)
    return np.array(keep, dtype=np.int32)
