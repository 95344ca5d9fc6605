"""Device-side plumbing shared by the parity tests and the benchmark: upload
one packed batch (arrays as produced by the `workloads` module), run the HIP
path through the binding (which calls the C ABI), fetch results as numpy.
Holds no arithmetic of the method and never touches the CPU checker."""
import numpy as np
import torch

from . import binding as pdd


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
        # scratch for the calls that can use one (partial importance sums: of the sweep inside the
        # attention kernel in chunked mode, else of the importance kernel's row split)
        desc, keep = pdd.make_desc(self.q, self.k, self.v, self.o, self.cu_q, self.cu_k, self.max_q, self.max_k,
                                   wl.scale, wl.window)
        call = pdd.CALL_PREFILL_ATTN_CHUNKED if wl.chunked else pdd.CALL_PREFILL_ATTN
        self.workspace_bytes = pdd.workspace_bytes(desc, call) if wl.total_k else 0
        self.workspace = (torch.empty(self.workspace_bytes, dtype=torch.uint8, device="cuda")
                          if self.workspace_bytes else None)
        del keep

    def poison(self):
        """Fill the outputs with junk so that an unwritten element shows."""
        self.o.view(torch.int16).fill_(0x7FC0)          # bf16 NaN
        self.lse.fill_(float("nan"))
        self.imp.fill_(float("nan"))
        self.idx.fill_(-7)
        self.mask.fill_(9)

    def attn(self, with_importance=True, host_cu=True, use_workspace=True):
        wl = self.wl
        hq = wl.cu_seqlens_q if host_cu else None
        hk = wl.cu_seqlens_k if host_cu else None
        # use_workspace: True = all of it, False = none, an int = only that many bytes of it
        ws = self.workspace if use_workspace else None
        if ws is not None and use_workspace is not True:
            ws = ws[:int(use_workspace)]
        if wl.chunked:
            pdd.prefill_attn_chunked(self.q, self.k, self.v, self.o, self.lse,
                                     self.imp if with_importance else None, self.cu_q, self.cu_k,
                                     self.max_q, self.max_k, wl.scale, hq, hk, workspace=ws)
        else:
            pdd.prefill_attn(self.q, self.k, self.v, self.o, self.lse,
                             self.imp if with_importance else None, self.cu_q, self.cu_k,
                             self.max_q, self.max_k, wl.scale,
                             wl.window if with_importance else 0, hq, hk, workspace=ws)

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
