"""Shared plumbing for the GPU parity tests: the device harness of the package
plus the comparison of selected index sets with the oracle's."""
import numpy as np

from paper_2508_09035_amd.harness import DeviceWorkload, bf16_dev, bf16_to_f64  # noqa: F401


def check_selection(scores64, got_idx, got_mask, wl, rel_tie, label=""):
    """Compare selected index sets per (head, sequence) with the oracle's
    selection on `scores64`; indices may differ only where the score is within
    rel_tie * |tau_k| of the k-th score tau_k (relative to the threshold itself,
    with a floor of 1e-12 for thresholds near zero); rel_tie < 0 allows nothing.
    Returns the number of swapped indices."""
    import oracle
    want_idx, want_mask = oracle.select_topk(scores64, wl.cu_seqlens_k, wl.k_keep,
                                             wl.cand_begin, wl.cand_end)
    cu_keep = wl.cu_keep
    swapped = 0
    for g in range(scores64.shape[0]):
        for b in range(wl.batch):
            got = got_idx[g, cu_keep[b]:cu_keep[b + 1]]
            want = want_idx[g, cu_keep[b]:cu_keep[b + 1]]
            assert len(got) < 2 or (np.diff(got) > 0).all(), f"{label}: indices not ascending"
            ks, ke = wl.cu_seqlens_k[b], wl.cu_seqlens_k[b + 1]
            m = got_mask[g, ks:ke]
            assert m.sum() == len(got) and (m[got] == 1).all() and set(np.unique(m)) <= {0, 1}, \
                f"{label}: mask does not match indices"
            assert ((got >= wl.cand_begin[b]) & (got < wl.cand_end[b])).all()
            if np.array_equal(got, want):
                continue
            row = scores64[g, ks:ke]
            tau = row[want].min()
            diff = np.setxor1d(got, want)
            tol = max(rel_tie * abs(tau), 1e-12) if rel_tie >= 0 else 0
            bad = [int(j) for j in diff if abs(row[j] - tau) > tol]
            assert not bad, f"{label}: head {g} seq {b}: indices {bad[:8]} differ beyond ties"
            swapped += len(diff)
    return swapped
