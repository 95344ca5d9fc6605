"""Shared plumbing for the GPU parity tests: upload a workload, run the HIP
path through the binding (which calls the C ABI), fetch results as numpy."""
import numpy as np
import torch

import paper_2508_09035_amd as pdd


def bf16_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def bf16_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


class DeviceWorkload:
    def __init__(self, wl):
        self.wl = wl
        self.q, self.k, self.v = bf16_dev(wl.q), bf16_dev(wl.k), bf16_dev(wl.v)
        self.cu_q = torch.from_numpy(wl.cu_seqlens_q).cuda()
        self.cu_k = torch.from_numpy(wl.cu_seqlens_k).cuda()
        self.max_q = int(wl.seqlens_q.max()) if wl.batch else 0
        self.max_k = int(wl.seqlens_k.max()) if wl.batch else 0
        self.o = torch.empty_like(self.q)
        self.lse = torch.empty((wl.n_q_heads, wl.total_q), dtype=torch.float32, device="cuda")
        self.imp = torch.empty((wl.n_kv_heads, wl.total_k), dtype=torch.float32, device="cuda")
        self.cand_b = torch.from_numpy(wl.cand_begin).cuda()
        self.cand_e = torch.from_numpy(wl.cand_end).cuda()
        self.k_keep = torch.from_numpy(wl.k_keep).cuda()
        self.cu_keep = torch.from_numpy(wl.cu_keep).cuda()
        self.total_keep = int(wl.cu_keep[-1])
        self.idx = torch.empty((wl.n_kv_heads, self.total_keep), dtype=torch.int32, device="cuda")
        self.mask = torch.empty((wl.n_kv_heads, wl.total_k), dtype=torch.uint8, device="cuda")

    def poison(self):
        """Fill the outputs with junk so that an unwritten element shows."""
        self.o.view(torch.int16).fill_(0x7FC0)          # bf16 NaN
        self.lse.fill_(float("nan"))
        self.imp.fill_(float("nan"))
        self.idx.fill_(-7)
        self.mask.fill_(9)

    def attn(self, with_importance=True, host_cu=True):
        wl = self.wl
        hq = wl.cu_seqlens_q if host_cu else None
        hk = wl.cu_seqlens_k if host_cu else None
        if wl.chunked:
            pdd.prefill_attn_chunked(self.q, self.k, self.v, self.o, self.lse,
                                     self.imp if with_importance else None, self.cu_q, self.cu_k,
                                     self.max_q, self.max_k, wl.scale, hq, hk)
        else:
            pdd.prefill_attn(self.q, self.k, self.v, self.o, self.lse,
                             self.imp if with_importance else None, self.cu_q, self.cu_k,
                             self.max_q, self.max_k, wl.scale,
                             wl.window if with_importance else 0, hq, hk)

    def select(self, scores=None):
        wl = self.wl
        pdd.select_topk(self.imp if scores is None else scores, self.cu_k, self.max_k,
                        self.k_keep, self.cu_keep, self.total_keep, self.idx, self.mask,
                        self.cand_b, self.cand_e, wl.cu_seqlens_k)

    def step(self):
        """One pass of the whole hot path."""
        self.attn(True)
        self.select()

    def results(self):
        torch.cuda.synchronize()
        return (bf16_to_f64(self.o), self.lse.cpu().numpy().astype(np.float64),
                self.imp.cpu().numpy().astype(np.float64), self.idx.cpu().numpy(),
                self.mask.cpu().numpy())


def check_selection(scores64, got_idx, got_mask, wl, rel_tie, label=""):
    """Compare selected index sets per (head, sequence) with the oracle's
    selection on `scores64`; indices may differ only where the score is within
    rel_tie * max(1, tau_k) of the k-th score tau_k.  Returns the number of
    swapped indices."""
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
            tol = rel_tie * max(1.0, abs(tau)) if rel_tie >= 0 else 0
            bad = [int(j) for j in diff if abs(row[j] - tau) > tol]
            assert not bad, f"{label}: head {g} seq {b}: indices {bad[:8]} differ beyond ties"
            swapped += len(diff)
    return swapped
