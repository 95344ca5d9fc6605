"""ctypes front end of the C oracle, plus the selection step in numpy.

Test infrastructure only (see the package docstring)."""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pdd_oracle.c")
_LIB = os.path.join(_HERE, "libpdd_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile pdd_oracle.c with gcc (generic x86-64, no fast-math, no FMA
    contraction) into libpdd_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.pddo_attention.restype = ctypes.c_int
        lib.pddo_attention.argtypes = [u16p, u16p, u16p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_int, i32p, i32p, ctypes.c_double, ctypes.c_int,
                                       i32p, f64p, f64p]
        lib.pddo_importance.restype = ctypes.c_int
        lib.pddo_importance.argtypes = [u16p, u16p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                        ctypes.c_int, i32p, i32p, ctypes.c_double, ctypes.c_int,
                                        f64p]
        lib.pddo_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().pddo_num_threads())


def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> float64, exactly."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _check_inputs(q, k, v, cu_q, cu_k):
    q = np.ascontiguousarray(q, dtype=np.uint16)
    k = np.ascontiguousarray(k, dtype=np.uint16)
    v = None if v is None else np.ascontiguousarray(v, dtype=np.uint16)
    cu_q = np.ascontiguousarray(cu_q, dtype=np.int32)
    cu_k = np.ascontiguousarray(cu_k, dtype=np.int32)
    assert q.ndim == 3 and k.ndim == 3 and q.shape[2] == k.shape[2]
    assert q.shape[0] == cu_q[-1] and k.shape[0] == cu_k[-1] and len(cu_q) == len(cu_k)
    if v is not None:
        assert v.shape == k.shape
    return q, k, v, cu_q, cu_k


def attention(q, k, v, cu_q, cu_k, scale: float, rows: Optional[Sequence[int]] = None):
    """O [n_rows, Hq, d] and LSE [Hq, n_rows] (float64) for the packed query
    rows `rows` (default: all)."""
    q, k, v, cu_q, cu_k = _check_inputs(q, k, v, cu_q, cu_k)
    B = len(cu_q) - 1
    Hq, d, Hkv = q.shape[1], q.shape[2], k.shape[1]
    if rows is None:
        rows_arr, n_rows, rows_ptr = None, q.shape[0], None
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int32)
        n_rows, rows_ptr = len(rows_arr), _ptr(rows_arr, ctypes.c_int32)
    O = np.empty((n_rows, Hq, d), dtype=np.float64)
    lse = np.empty((Hq, n_rows), dtype=np.float64)
    rc = _load().pddo_attention(_ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16),
                                _ptr(v, ctypes.c_uint16), B, Hq, Hkv, d,
                                _ptr(cu_q, ctypes.c_int32), _ptr(cu_k, ctypes.c_int32),
                                float(scale), n_rows, rows_ptr,
                                _ptr(O, ctypes.c_double), _ptr(lse, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle attention: bad arguments")
    return O, lse


def importance(q, k, cu_q, cu_k, scale: float, window: int) -> np.ndarray:
    """imp [Hkv, total_k] float64.  window < 0: every query is a window query."""
    q, k, _, cu_q, cu_k = _check_inputs(q, k, None, cu_q, cu_k)
    B = len(cu_q) - 1
    Hq, d, Hkv = q.shape[1], q.shape[2], k.shape[1]
    imp = np.empty((Hkv, k.shape[0]), dtype=np.float64)
    rc = _load().pddo_importance(_ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16),
                                 B, Hq, Hkv, d, _ptr(cu_q, ctypes.c_int32),
                                 _ptr(cu_k, ctypes.c_int32), float(scale), int(window),
                                 _ptr(imp, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle importance: bad arguments")
    return imp


def select_topk(scores: np.ndarray, cu_k, k_per_seq, cand_begin=None, cand_end=None):
    """Top-k selection per (KV head, sequence).

    Candidates of sequence b are its keys [cand_begin[b], cand_end[b]) (default:
    all).  They are ordered by (score descending, index ascending); the first
    k_per_seq[b] are kept and reported in ascending index order
    (sequence-local).  Returns (indices [Hkv, sum k], mask uint8 [Hkv, total_k]).
    """
    scores = np.asarray(scores)
    cu_k = np.asarray(cu_k, dtype=np.int64)
    B = len(cu_k) - 1
    Hkv = scores.shape[0]
    k_per_seq = np.asarray(k_per_seq, dtype=np.int64)
    cu_keep = np.concatenate([[0], np.cumsum(k_per_seq)])
    idx_out = np.zeros((Hkv, int(cu_keep[-1])), dtype=np.int32)
    mask = np.zeros((Hkv, int(cu_k[-1])), dtype=np.uint8)
    for g in range(Hkv):
        for b in range(B):
            n = int(cu_k[b + 1] - cu_k[b])
            c0 = 0 if cand_begin is None else int(cand_begin[b])
            c1 = n if cand_end is None else int(cand_end[b])
            kb = int(k_per_seq[b])
            if not (0 <= c0 <= c1 <= n) or kb > c1 - c0 or kb < 0:
                raise ValueError("bad candidate range or k")
            cand = np.arange(c0, c1)
            s = scores[g, cu_k[b] + c0: cu_k[b] + c1]
            order = np.lexsort((cand, -s))          # primary: -score, then index
            keep = np.sort(cand[order[:kb]])
            idx_out[g, cu_keep[b]:cu_keep[b + 1]] = keep
            mask[g, cu_k[b] + keep] = 1
    return idx_out, mask


def pack_mask(mask: np.ndarray, cu_k):
    """Mask -> bit stream per (row, sequence), byte aligned, first token in the
    most significant bit (Section 3.2: the mask is treated as a bit stream).
    Returns (bits uint8 [rows, sum ceil(n_b/8)], cu_bytes)."""
    mask = np.asarray(mask, dtype=np.uint8)
    cu_k = np.asarray(cu_k, dtype=np.int64)
    nbytes = [(int(cu_k[b + 1] - cu_k[b]) + 7) // 8 for b in range(len(cu_k) - 1)]
    cu_bytes = np.concatenate([[0], np.cumsum(nbytes)]).astype(np.int32)
    out = np.zeros((mask.shape[0], int(cu_bytes[-1])), dtype=np.uint8)
    for r in range(mask.shape[0]):
        for b in range(len(cu_k) - 1):
            seg = (mask[r, cu_k[b]:cu_k[b + 1]] != 0).astype(np.uint8)
            out[r, cu_bytes[b]:cu_bytes[b + 1]] = np.packbits(seg)   # bitorder 'big'
    return out, cu_bytes


def pool_scores(scores: np.ndarray, cu_k, kernel: int, mode: str) -> np.ndarray:
    """1-D pooling of the summed scores along each sequence before sorting
    (Section 3.2 "Prompt Refiner": a pooling step that clusters neighbouring tokens).
    Window of key j: keys [j - r, j + r] of the same sequence, r = (kernel-1)/2.
    mode "max": maximum over the part of the window inside the sequence;
    mode "avg": sum over that part divided by `kernel` (zero padding).
    The paper states neither size nor type; both are parameters."""
    scores = np.asarray(scores, dtype=np.float64)
    cu_k = np.asarray(cu_k, dtype=np.int64)
    assert kernel >= 1 and kernel % 2 == 1 and mode in ("max", "avg")
    r = (kernel - 1) // 2
    out = np.empty_like(scores)
    for g in range(scores.shape[0]):
        for b in range(len(cu_k) - 1):
            seq = scores[g, cu_k[b]:cu_k[b + 1]]
            n = len(seq)
            for j in range(n):
                win = seq[max(0, j - r):min(n, j + r + 1)]
                out[g, cu_k[b] + j] = win.max() if mode == "max" else win.sum() / kernel
    return out


def select_sentences(scores, cu_k, cu_sent, sent_end, token_budget, mode="mean", cand_begin=None,
                     sum_dtype=np.float64):
    """Sentence-level selection (Section 3.2 "Prompt Refiner": the KV cache of one
    sentence is treated as a whole, so selection means selecting sentences).
    Sentence s of sequence b covers tokens [start, sent_end[s]), start = cand_begin[b]
    for the first sentence, else the previous end.  Score = sum (or mean) of the
    token scores, added in token order in `sum_dtype`; sentences ranked by (score
    descending, index ascending); the longest ranking prefix whose token count is
    <= token_budget[b] is kept.
    Returns (sent_scores [H,total_sent], sent_keep uint8 [H,total_sent],
    mask uint8 [H,total_k], kept_tokens int32 [H,B])."""
    scores = np.asarray(scores)
    cu_k = np.asarray(cu_k, dtype=np.int64)
    cu_sent = np.asarray(cu_sent, dtype=np.int64)
    sent_end = np.asarray(sent_end, dtype=np.int64)
    H, B = scores.shape[0], len(cu_k) - 1
    sscore = np.zeros((H, len(sent_end)), dtype=np.float64)
    skeep = np.zeros((H, len(sent_end)), dtype=np.uint8)
    mask = np.zeros((H, int(cu_k[-1])), dtype=np.uint8)
    kept = np.zeros((H, B), dtype=np.int32)
    for g in range(H):
        for b in range(B):
            n = int(cu_k[b + 1] - cu_k[b])
            c0 = 0 if cand_begin is None else int(cand_begin[b])
            ends = sent_end[cu_sent[b]:cu_sent[b + 1]]
            starts = np.concatenate([[c0], ends[:-1]]) if len(ends) else ends
            assert all(0 <= s <= e <= n for s, e in zip(starts, ends))
            vals = []
            for s, e in zip(starts, ends):
                acc = sum_dtype(0)
                for x in range(int(s), int(e)):
                    acc = sum_dtype(acc + sum_dtype(scores[g, cu_k[b] + x]))
                if mode == "mean":
                    acc = sum_dtype(acc / sum_dtype(max(int(e - s), 1)))
                vals.append(float(acc))
            vals = np.array(vals, dtype=np.float64)
            sscore[g, cu_sent[b]:cu_sent[b + 1]] = vals
            order = np.lexsort((np.arange(len(vals)), -vals))
            total = 0
            for s in order:
                ln = int(ends[s] - starts[s])
                if total + ln > int(token_budget[b]):
                    break
                total += ln
                skeep[g, cu_sent[b] + s] = 1
                mask[g, cu_k[b] + starts[s]: cu_k[b] + ends[s]] = 1
            kept[g, b] = total
    return sscore, skeep, mask, kept


def aggregate_scores(scores, weights=None, reduce_heads=False, acc=None):
    """Weighted sum of per-layer importance scores [L, H, N] over layers, and over
    heads when reduce_heads (Section 4.4: several attention layers take part in
    the selection; the strategy is left open, so the weights are inputs).  fp64.
    acc: previous contents of the output when accumulating."""
    s = np.asarray(scores, dtype=np.float64)
    w = np.ones(s.shape[0]) if weights is None else np.asarray(weights, dtype=np.float64)
    out = np.zeros((1 if reduce_heads else s.shape[1], s.shape[2]))
    for l in range(s.shape[0]):
        for h in range(s.shape[1]):
            out[0 if reduce_heads else h] += w[l] * s[l, h]
    return out if acc is None else out + np.asarray(acc, dtype=np.float64)


def choose_r_L(l, k_c, k_d, delta, xi_scene, tpot_c, tpot_d, tau, delta_cloud=0.0, r_grid=2000,
               L_max=5000):
    """Program P of Section 3.4 ("Algorithm on Refiner and Termination") by exhaustive
    search in exact rational arithmetic: minimise TTFT_d over candidate ratios r in [0, 1]
    and integers 2 <= L <= L_max.
      Eq. 2:  TTFT_c = prefill_c(l) + compress + RTT       = k_c l + delta_cloud
      Eq. 3:  TTFT_d = TTFT_c + decompress + prefill_d(rl) = k_c l + delta + k_d r l
    with delta the bound on compress + decompress + RTT and delta_cloud its part spent before
    the first token reaches the device (compress + RTT), 0 <= delta_cloud <= delta.
    Subject to Eq. 5 (xi_scene <= r <= 1 - (k_c + delta/l)/k_d) and Eq. 6
    ((prefill_d(rl) - TTFT_c)/(tau - TPOT_d) <= L-1 <= (TTFT_d - TTFT_c)/TPOT_c).
    r is a real number, so besides a uniform grid and xi_scene the candidates include every
    ratio at which the cloud-occupation bound of Eq. 6 becomes tight for an integer L (the
    only other places where the feasible set can start).  Among minimisers the smallest L is
    returned (Section 4.2: the optimum is at L's lower bound).  Returns (r, L) with r a
    float, or None when nothing is feasible."""
    from fractions import Fraction as F
    from math import ceil
    l, k_c, k_d, delta, xi, tpot_c, tpot_d, tau, d_c = (
        F(x) for x in (l, k_c, k_d, delta, xi_scene, tpot_c, tpot_d, tau, delta_cloud))
    assert 0 <= d_c <= delta and tau > tpot_d
    cands = {F(i, r_grid) for i in range(r_grid + 1)} | {xi}
    cands |= {((L - 1) * tpot_c - (delta - d_c)) / (k_d * l) for L in range(2, L_max + 1)}
    best = None
    for r in sorted(c for c in cands if 0 <= c <= 1):
        if not (xi <= r <= 1 - (k_c + delta / l) / k_d):
            continue
        ttft_c = k_c * l + d_c
        ttft_d = ttft_c + (delta - d_c) + k_d * r * l
        lo = (k_d * r * l - ttft_c) / (tau - tpot_d)          # smoothed-TPOT bound on L - 1
        hi = (ttft_d - ttft_c) / tpot_c                       # cloud-occupation bound on L - 1
        L = max(2, ceil(lo) + 1)                              # smallest integer L > 1 with L - 1 >= lo
        if L - 1 <= hi and L <= L_max and (best is None or ttft_d < best[0]):
            best = (ttft_d, r, L)
    return None if best is None else (float(best[1]), best[2])
