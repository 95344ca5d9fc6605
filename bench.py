"""Benchmark of the hot path on one MI355X.

One "step" = one pass of the whole path over one synthetic batch: fused causal
prefill attention + observation-window importance, then top-k selection with
index compaction.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line (see the field notes at the bottom of this file).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch of the attention kernel (FETCH_SIZE + WRITE_SIZE of rocprofv3 --pmc runs, each
# scaled by the same counter's reading for a 1 GiB device copy; see profiles/).  Valid only for the
# kernel sources with this digest: once they change the figure is reported as null.
KERNEL_SOURCES = ("attn_fwd_d128.hpp", "attn_fwd.hpp")
TRAFFIC = {"c4": {"bytes": 1.679e9, "sources_sha256": "1009c1eeac8510839fc7860fac20275dbe402f28f8df4b6574fd7eb6dd409668"}}


def kernel_digest():
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2508_09035_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def time_gpu(fn, iters, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / iters     # ms


def cpu_baseline(wl, budget_gflop=200.0):
    """Time the oracle (as it stands) on a bounded seeded sample of query rows
    of the same workload, on the host cores."""
    import numpy as np
    import oracle
    d, hq = wl.head_dim, wl.n_q_heads
    rng = np.random.default_rng(1234)
    rows, flops = [], 0.0
    total_q = wl.total_q
    order = rng.permutation(total_q)
    cu_q, cu_k = wl.cu_seqlens_q, wl.cu_seqlens_k
    for r in order:
        b = int(np.searchsorted(cu_q, r, side="right") - 1)
        i = int(r - cu_q[b])
        n_vis = i + int((cu_k[b + 1] - cu_k[b]) - (cu_q[b + 1] - cu_q[b])) + 1
        rows.append(int(r))
        flops += 4.0 * d * hq * n_vis
        if flops >= budget_gflop * 1e9:
            break
    rows = np.array(sorted(rows), dtype=np.int32)
    t0 = time.perf_counter()
    oracle.attention(wl.q, wl.k, wl.v, cu_q, cu_k, wl.scale, rows=rows)
    dt = time.perf_counter() - t0
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"{len(rows)} seeded random query rows x {hq} heads of {wl.name} "
                      f"({flops / 1e9:.1f} GFLOP of attention, fp64, {dt:.1f} s)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="c4", help="workload: c1..c5 (default: the 32k-token prompt)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--waves", type=int, default=0, help="attention waves per workgroup (0 = auto)")
    ap.add_argument("--kernel-digest", action="store_true", help="print the digest of the attention "
                    "kernel sources (the key of the stored HBM traffic figure) and exit")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="after the timed legs also run one plain device copy of this many MiB "
                         "(a known-size reference for HBM byte counters)")
    args = ap.parse_args()
    if args.kernel_digest:
        print(kernel_digest())
        return
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads
    import paper_2508_09035_amd as pdd
    from gpu_harness import DeviceWorkload

    pdd.load_library()                      # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    wl = workloads.make_workload(args.config)
    dev = DeviceWorkload(wl)
    pdd.set_option(pdd.OPT_ATTN_WAVES, args.waves)

    # whole path
    ms_step = time_gpu(dev.step, args.steps, args.warmup)
    # per-kernel legs (same launch configuration), HIP events on the launch stream
    ms_attn = time_gpu(lambda: dev.attn(with_importance=False), args.steps, 2)
    ms_attn_imp = time_gpu(lambda: dev.attn(with_importance=True), args.steps, 2)
    ms_select = time_gpu(dev.select, args.steps, 2)

    if args.calibration_copy_mib > 0:
        src = torch.ones(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    attn_flops, imp_flops = wl.attn_flops(), wl.importance_flops()
    tflops_path = (attn_flops + imp_flops) / (ms_step * 1e-3) / 1e12
    tflops_attn = attn_flops / (ms_attn * 1e-3) / 1e12
    sel_bytes = 4 * wl.n_kv_heads * int((wl.cand_end - wl.cand_begin).sum()) \
        + 4 * wl.n_kv_heads * int(wl.k_keep.sum()) + wl.n_kv_heads * wl.total_k
    t = TRAFFIC.get(wl.name)
    traffic = t["bytes"] if t and t["sources_sha256"] == kernel_digest() else None
    out = {
        "metric": "causal prefill attn TFLOP/s (+importance) & % bf16 MFMA peak; prompt tokens/s",
        "value": round(tflops_path, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.notes}", "batch": wl.batch,
                   "total_q": wl.total_q, "total_k": wl.total_k, "n_q_heads": wl.n_q_heads,
                   "n_kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim, "window": wl.window,
                   "keep_ratio": str(wl.keep_ratio), "parallelism": "single GPU"},
        "pct_bf16_mfma_peak": round(100 * tflops_path / PEAK_BF16_TFLOPS, 2),
        "prompt_tokens_per_s": round(wl.total_q / (ms_step * 1e-3), 1),
        "legs_ms": {"attention": round(ms_attn, 4), "attention+importance": round(ms_attn_imp, 4),
                    "select+compaction": round(ms_select, 4)},
        "select_GBps": round(sel_bytes / (ms_select * 1e-3) / 1e9, 2),
        "roofline": {"bound": "mfma",
                     "kernel": "attn_fwd_d128_kernel" if wl.head_dim == 128 else "attn_fwd_kernel",
                     "achieved": round(tflops_attn, 2), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(tflops_attn / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

# Field notes
#   value / unit   whole-path throughput: (attention + importance flops, causal-halved,
#                  4*d per visible pair + 2*d per window pair) / step time
#   roofline       the attention kernel alone: algorithmic flops per launch / its
#                  average duration between HIP events, against the dense bf16 MFMA peak
#                  traffic = HBM bytes per launch from byte counters (null when not measured for
#                  these kernel sources)
#   cpu_baseline   the fp64 oracle timed on a bounded sample of rows (reported, not a target)
