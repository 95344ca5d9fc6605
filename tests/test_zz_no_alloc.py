"""The chunked entry point that allocates nothing (it keeps its scratch in an array inside the
library's device image) against the ordinary chunked entry point with a caller workspace:
identical bits, on two calls in a row, the second on a smaller input."""
import numpy as np
import pytest
import torch

import workloads as W
import paper_2508_09035_amd as pdd
from gpu_harness import DeviceWorkload

pytestmark = pytest.mark.gpu


def _both_ways(wl):
    dev = DeviceWorkload(wl)
    assert dev.workspace_bytes > 0, "the shape must be one that uses scratch"
    dev.poison()
    dev.attn(True)                                  # pdd_prefill_attn_chunked with the caller's workspace
    torch.cuda.synchronize()
    want = [x.clone() for x in (dev.o, dev.lse, dev.imp)]
    dev.poison()
    before = torch.cuda.memory_allocated()
    pdd.prefill_attn_chunked_noalloc(dev.q, dev.k, dev.v, dev.o, dev.lse, dev.imp, dev.cu_q, dev.cu_k,
                                     dev.max_q, dev.max_k, wl.scale, wl.cu_seqlens_q, wl.cu_seqlens_k)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for name, a, b in zip(("O", "lse", "importance"), want, (dev.o, dev.lse, dev.imp)):
        assert torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a.view(torch.int16),
                           b.view(torch.int32) if b.dtype == torch.float32 else b.view(torch.int16)), name
    assert np.isfinite(dev.imp.cpu().numpy()).all()


def test_noalloc_chunked_matches_workspace_call_twice():
    _both_ways(W.make_workload("c5"))               # 4 x (8192 + 256) keys, 64 / 8 heads
    _both_ways(W.make_custom("t", [200, 256], [200 + 5000, 256 + 6000], 32, 2, 128, 0, "1/4",
                             seed=43, chunked=True))


def test_noalloc_chunked_under_graph_capture():
    """What the entry point is for: the chunked call and the selection behind it captured in a HIP
    graph (nothing in them allocates, frees or clears memory) and replayed three times, with eager
    work and a synchronisation between the replays; every replay gives the eager run's bits."""
    wl = W.make_workload("c5")
    dev = DeviceWorkload(wl)

    def path():
        pdd.prefill_attn_chunked_noalloc(dev.q, dev.k, dev.v, dev.o, dev.lse, dev.imp, dev.cu_q, dev.cu_k,
                                         dev.max_q, dev.max_k, wl.scale, wl.cu_seqlens_q, wl.cu_seqlens_k)
        dev.select()

    path()                                          # eager; also looks up the scratch address once
    torch.cuda.synchronize()
    want = [x.clone() for x in (dev.o, dev.lse, dev.imp, dev.idx, dev.mask)]
    side = torch.cuda.Stream()                      # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        path()                                      # once on the stream that will be captured
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        path()
    torch.cuda.synchronize()
    for rep in range(3):
        dev.poison()
        torch.randn(1 << 20, device="cuda").sum().item()
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("O", "lse", "importance", "indices", "mask"), want,
                              (dev.o, dev.lse, dev.imp, dev.idx, dev.mask)):
            assert torch.equal(a, b), f"replay {rep}: {name}"
