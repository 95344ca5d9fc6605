"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2508_09035_amd as pdd
from paper_2508_09035_amd.binding import AttnDesc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "pdd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pdd_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = pdd.load_library()
    names = header_functions()
    assert {"pdd_prefill_attn", "pdd_prefill_attn_chunked", "pdd_token_importance",
            "pdd_select_topk", "pdd_workspace_bytes", "pdd_last_error"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    assert "gfx950" in pdd.version()


def good_desc():
    d = AttnDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim = 1, 4, 2, 128
    d.total_q = d.total_k = d.max_seqlen_q = d.max_seqlen_k = 64
    d.cu_seqlens_q = d.cu_seqlens_k = 0x1000          # fake device addresses, never followed
    for f in ("q", "k", "v", "o"):
        heads = 4 if f in "qo" else 2
        setattr(d, f + "_stride_tok", heads * 128)
        setattr(d, f + "_stride_head", 128)
    d.window = 8
    return d


def call_prefill(d, q=0x10000, k=0x20000, v=0x30000, o=0x40000, lse=0x50000, imp=0x60000):
    return pdd.load_library().pdd_prefill_attn(ctypes.byref(d), q, k, v, o, lse, imp, None, 0, None)


@pytest.mark.parametrize("mutate,status,needle", [
    (lambda d: setattr(d, "n_kv_heads", 3), -1, "n_q_heads"),
    (lambda d: setattr(d, "head_dim", 96), -2, "head_dim"),
    (lambda d: setattr(d, "batch", 0), -1, "batch"),
    (lambda d: setattr(d, "cu_seqlens_q", None), -1, "cu_seqlens"),
    (lambda d: setattr(d, "q_stride_tok", 100), -1, "stride"),
    (lambda d: setattr(d, "k_stride_head", 132), -1, "multiple of 8"),
    (lambda d: setattr(d, "window", -1), -1, "window"),
    (lambda d: setattr(d, "total_k", 65), -1, "total_q == total_k"),
    (lambda d: setattr(d, "max_seqlen_q", 65), -1, "max_seqlen"),
])
def test_descriptor_validation(mutate, status, needle):
    d = good_desc()
    mutate(d)
    assert call_prefill(d) == status
    assert needle in pdd.load_library().pdd_last_error().decode()


def test_pointer_validation():
    d = good_desc()
    assert call_prefill(d, q=None) == -1
    assert call_prefill(d, v=0x30008) == -1                     # misaligned
    assert call_prefill(d, imp=None) == -1                      # window > 0 needs importance
    assert "importance" in pdd.load_library().pdd_last_error().decode()


def test_host_cu_seqlens_validation():
    lib = pdd.load_library()
    d = good_desc()
    for bad, needle in [([1, 64], "[0] must be 0"), ([0, 63], "differs from the total"),
                        ([0, 70], "longer than max_seqlen")]:
        arr = np.array(bad, dtype=np.int32)
        d.cu_seqlens_q_host = arr.ctypes.data
        assert call_prefill(d) == -1
        assert needle in lib.pdd_last_error().decode()
    d = good_desc()
    d.batch = 2
    arr = np.array([0, 40, 30], dtype=np.int32)
    d.cu_seqlens_k_host = arr.ctypes.data
    assert call_prefill(d) == -1 and "non-decreasing" in lib.pdd_last_error().decode()
    # chunked: fewer keys than queries in one sequence
    d = good_desc()
    d.batch, d.total_q, d.total_k, d.max_seqlen_k = 2, 64, 80, 60
    aq = np.array([0, 40, 64], dtype=np.int32)
    ak = np.array([0, 20, 80], dtype=np.int32)
    d.cu_seqlens_q_host, d.cu_seqlens_k_host = aq.ctypes.data, ak.ctypes.data
    rc = lib.pdd_prefill_attn_chunked(ctypes.byref(d), 0x10000, 0x20000, 0x30000, 0x40000,
                                      0x50000, None, None, 0, None)
    assert rc == -1 and "fewer keys" in lib.pdd_last_error().decode()


def test_importance_and_select_validation():
    lib = pdd.load_library()
    d = good_desc()
    d.window = 0
    assert lib.pdd_token_importance(ctypes.byref(d), 0x10000, 0x20000, 0x50000, 0x60000,
                                    None, 0, None) == -1
    sel = lambda **kw: lib.pdd_select_topk(
        kw.get("scores", 0x1000), kw.get("heads", 2), kw.get("batch", 1), kw.get("total_k", 64),
        kw.get("cu", 0x2000), None, kw.get("max_k", 64), kw.get("cb", None), kw.get("ce", None),
        kw.get("kper", 0x3000), kw.get("cukeep", 0x4000), kw.get("total_keep", 8),
        kw.get("out", 0x5000), None, None, 0, None)
    assert sel(scores=None) == -1
    assert sel(heads=0) == -1
    assert sel(max_k=65) == -1
    assert sel(out=None) == -1
    assert sel(cb=0x6000) == -1 and "both" in lib.pdd_last_error().decode()
    assert pdd.set_option(pdd.OPT_ATTN_WAVES, 8) is None
    with pytest.raises(pdd.PddError):
        pdd.set_option(pdd.OPT_ATTN_WAVES, 5)
    pdd.set_option(pdd.OPT_ATTN_WAVES, 0)
    assert pdd.set_option(pdd.OPT_IMPORTANCE_KEYS, 128) is None
    with pytest.raises(pdd.PddError):
        pdd.set_option(pdd.OPT_IMPORTANCE_KEYS, 64)
    pdd.set_option(pdd.OPT_IMPORTANCE_KEYS, 0)
    with pytest.raises(pdd.PddError):
        pdd.set_option(7, 0)
    assert pdd.workspace_bytes(good_desc(), 0) < 64 * 64 * 4     # never O(N^2)


def test_choose_r_L_against_exhaustive_search():
    """Host-only entry point: the closed form must agree with the oracle's search of program P."""
    import oracle
    rng = np.random.default_rng(5)
    n_feasible = n_infeasible = n_moved = 0
    for it in range(100):
        if it < 60:         # long prompts: the quality bound xi_scene is the optimum whenever P is feasible
            c = dict(l=int(rng.integers(64, 40000)), k_c=float(rng.uniform(0.005, 0.2)),
                     k_d=float(rng.uniform(0.1, 1.0)), delta=float(rng.uniform(0, 800)),
                     xi_scene=float(rng.integers(1, 19)) / 20, tpot_c=float(rng.uniform(10, 60)),
                     tpot_d=float(rng.uniform(30, 90)), tau=float(rng.uniform(95, 200)))
        else:               # short prompts: the cloud-occupation bound often pushes r above xi_scene
            c = dict(l=int(rng.integers(40, 400)), k_c=float(rng.uniform(0.005, 0.1)),
                     k_d=float(rng.uniform(0.3, 1.0)), delta=float(rng.uniform(0, 10)),
                     xi_scene=float(rng.integers(1, 8)) / 20, tpot_c=float(rng.uniform(10, 60)),
                     tpot_d=float(rng.uniform(30, 90)), tau=float(rng.uniform(95, 200)))
        c["delta_cloud"] = float(rng.uniform(0, 1)) * c["delta"] if rng.random() < 0.7 else 0.0
        want = oracle.choose_r_L(**c, L_max=8000 if it < 60 else 1000)
        if want is None:
            with pytest.raises(pdd.PddError) as e:
                pdd.choose_r_L(**c)
            assert e.value.status == -5
            n_infeasible += 1
        else:
            got = pdd.choose_r_L(**c)
            assert got[1] == want[1] and abs(got[0] - want[0]) <= 1e-12 * want[0]
            n_feasible += 1
            n_moved += want[0] > c["xi_scene"] * (1 + 1e-9)
    assert n_feasible >= 10 and n_infeasible >= 5 and n_moved >= 3
    with pytest.raises(pdd.PddError) as e:
        pdd.choose_r_L(0, 0.02, 0.5, 300, 0.6, 30, 50, 100)
    assert e.value.status == -1
    with pytest.raises(pdd.PddError) as e:                        # delta_cloud is a part of delta
        pdd.choose_r_L(100, 0.02, 0.5, 300, 0.6, 30, 50, 100, delta_cloud=301)
    assert e.value.status == -1
    # the split of delta decides feasibility (hand-worked in the oracle's pins)
    tight = dict(l=100, k_c=0.3, k_d=0.5, delta=5, xi_scene=0.2, tpot_c=12, tpot_d=50, tau=100)
    assert pdd.choose_r_L(**tight) == (0.2, 2)
    r, L = pdd.choose_r_L(**tight, delta_cloud=5)                 # xi_scene infeasible, 0.24 is the optimum
    assert abs(r - 0.24) < 1e-15 and L == 2
    with pytest.raises(pdd.PddError) as e:
        pdd.choose_r_L(**dict(tight, tpot_c=16), delta_cloud=5)
    assert e.value.status == -5
    assert pdd.choose_r_L(8192, 0.02, 0.5, 300, 0.6, 30, 50, 100, delta_cloud=200) == (0.6, 43)
    with pytest.raises(pdd.PddError) as e:                        # tau must exceed the device TPOT
        pdd.choose_r_L(100, 0.02, 0.5, 300, 0.6, 30, 50, 50)
    assert e.value.status == -5


def test_refinement_entry_points_validation():
    """Pooled selection, sentence selection, bit packing, aggregation: bad arguments are
    rejected on the host before anything is launched."""
    lib = pdd.load_library()
    pooled = lambda kernel, mode: lib.pdd_select_topk_pooled(
        0x1000, 2, 1, 64, 0x2000, None, 64, None, None, 0x3000, 0x4000, 8, kernel, mode, None,
        0x5000, None, None, 0, None)
    assert pooled(4, 1) == -1                      # even kernel
    assert pooled(3, 7) == -1                      # unknown mode
    sent = lambda **kw: lib.pdd_select_sentences(
        kw.get("scores", 0x1000), 2, 1, 64, 0x2000, None, 64, kw.get("cu_sent", 0x3000),
        kw.get("sent_end", 0x4000), kw.get("total_sent", 10), kw.get("max_sent", 10), None,
        kw.get("budget", 0x5000), kw.get("mode", 0), None, 0x6000, 0x7000, None, None)
    assert sent(scores=None) == -1
    assert sent(budget=None) == -1
    assert sent(mode=2) == -1
    assert sent(max_sent=11) == -1                 # more per sequence than in total
    assert sent(total_sent=20000, max_sent=9000) == -2 and "8192" in lib.pdd_last_error().decode()
    pack = lambda **kw: lib.pdd_pack_mask(kw.get("mask", 0x1000), 2, 1, 64, 0x2000, None,
                                          kw.get("max_k", 64), 0x3000, 8, kw.get("out", 0x4000), None)
    assert pack(mask=None) == -1
    assert pack(out=None) == -1
    assert pack(max_k=65) == -1
    agg = lambda **kw: lib.pdd_aggregate_scores(kw.get("scores", 0x1000), kw.get("layers", 2), 4, 64,
                                                kw.get("stride", 256), None, 0, 0, kw.get("out", 0x2000), None)
    assert agg(scores=None) == -1
    assert agg(out=None) == -1
    assert agg(layers=0) == -1
    assert agg(stride=255) == -1 and "layer_stride" in lib.pdd_last_error().decode()


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only; asking for more exits with a message instead of a JSON line."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_pack_mask_layout_matches_the_oracle_layout():
    import oracle
    cu = np.array([0, 13, 77, 77, 1077, 1084, 5183], dtype=np.int32)
    got, total = pdd.pack_mask_layout(cu)
    _, want = oracle.pack_mask(np.zeros((1, int(cu[-1])), dtype=np.uint8), cu)
    assert np.array_equal(got, want) and total == int(want[-1]) == sum((int(n) + 7) // 8 for n in np.diff(cu))
    with pytest.raises(pdd.PddError):
        pdd.pack_mask_layout(np.array([0, 5, 3], dtype=np.int32))


def test_workspace_bytes_host_only():
    """The scratch size is a pure function of the descriptor (and the device's compute-unit count,
    256 when no device is visible): 0 where the importance step is not divided, otherwise a whole
    number of [n_kv_heads, total_k] fp32 planes, at most 8."""
    lib = pdd.load_library()
    d = good_desc()                                     # 64 tokens, window 8: a single row block
    assert lib.pdd_workspace_bytes(ctypes.byref(d), 0) == 0
    d = good_desc()                                     # chunked catch-up shape: 4 x (8192 + 256) keys, 64/8 heads
    d.batch, d.n_q_heads, d.n_kv_heads = 4, 64, 8
    d.total_q, d.max_seqlen_q, d.total_k, d.max_seqlen_k = 1024, 256, 4 * 8448, 8448
    plane = 8 * 4 * 8448 * 4
    for call in (1, 2):
        d.window = -1
        n = lib.pdd_workspace_bytes(ctypes.byref(d), call)
        assert n > 0 and n % plane == 0 and n // plane <= 8
    assert lib.pdd_workspace_bytes(ctypes.byref(d), 3) == 0          # the selection uses none
    assert lib.pdd_workspace_bytes(None, 0) == 0
    # the chunked call asks for the sweep's room: one float per query head, 256-row query tile and key
    assert lib.pdd_workspace_bytes(ctypes.byref(d), 1) == 64 * 1 * 4 * 8448 * 4
    # ... unless that would pass 256 MiB: then it is the row split of the separate kernel again
    d.n_q_heads, d.total_q, d.max_seqlen_q = 128, 4 * 4096, 4096    # 128 heads x 16 query tiles x 33792 keys x 4 B
    n = lib.pdd_workspace_bytes(ctypes.byref(d), 1)
    assert 0 < n <= 8 * plane


def test_noalloc_rejects_shapes_beyond_its_scratch():
    """The allocation-free chunked entry point refuses, on the host, a shape whose scratch
    would not fit its built-in 16 MiB array: nothing is launched."""
    d = AttnDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim = 4, 128, 8, 128     # 16 query heads per KV head, chunks of 1024
    d.total_q, d.max_seqlen_q, d.total_k, d.max_seqlen_k = 4 * 1024, 1024, 4 * 8448, 8448
    d.cu_seqlens_q = d.cu_seqlens_k = 0x1000          # never followed: validation fails first
    for f in ("q", "k", "v", "o"):
        heads = 128 if f in "qo" else 8
        setattr(d, f + "_stride_tok", heads * 128)
        setattr(d, f + "_stride_head", 128)
    lib = pdd.load_library()
    assert lib.pdd_workspace_bytes(ctypes.byref(d), pdd.CALL_PREFILL_ATTN_CHUNKED) > (4 << 20)
    rc = lib.pdd_prefill_attn_chunked_noalloc(ctypes.byref(d), 0x10000, 0x20000, 0x30000, 0x40000, 0x50000,
                                              0x60000, None)
    assert rc == -3 and "scratch" in lib.pdd_last_error().decode()
