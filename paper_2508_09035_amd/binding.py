"""ctypes binding of libpdd.so: same names as the C entry points, argument
marshalling only.  Tensors are torch tensors on the GPU; raw `data_ptr()`s and
the current stream are handed to the library."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG_DIR, "libpdd.so")
_lib = None

OPT_ATTN_WAVES = 0
OPT_IMPORTANCE_KEYS = 1
CALL_PREFILL_ATTN, CALL_PREFILL_ATTN_CHUNKED, CALL_TOKEN_IMPORTANCE, CALL_SELECT_TOPK = 0, 1, 2, 3


class PddError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"pdd status {status}: {message}")
        self.status = status


class RLModel(ctypes.Structure):
    """Mirror of pdd_rl_model."""
    _fields_ = [(n, ctypes.c_double) for n in
                ("k_c", "k_d", "delta", "xi_scene", "tpot_c", "tpot_d", "tau", "delta_cloud")]


class AttnDesc(ctypes.Structure):
    """Mirror of `pdd_attn_desc`."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("total_q", ctypes.c_int32), ("total_k", ctypes.c_int32),
        ("max_seqlen_q", ctypes.c_int32), ("max_seqlen_k", ctypes.c_int32),
        ("cu_seqlens_q", ctypes.c_void_p), ("cu_seqlens_k", ctypes.c_void_p),
        ("cu_seqlens_q_host", ctypes.c_void_p), ("cu_seqlens_k_host", ctypes.c_void_p),
        ("q_stride_tok", ctypes.c_int64), ("q_stride_head", ctypes.c_int64),
        ("k_stride_tok", ctypes.c_int64), ("k_stride_head", ctypes.c_int64),
        ("v_stride_tok", ctypes.c_int64), ("v_stride_head", ctypes.c_int64),
        ("o_stride_tok", ctypes.c_int64), ("o_stride_head", ctypes.c_int64),
        ("softmax_scale", ctypes.c_float), ("window", ctypes.c_int32),
    ]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libpdd.so (built by `paper_2508_09035_amd.build.build_library`).
    Raises if it is missing: there is no other execution path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise PddError(-100, f"{_LIB_PATH} is not built; run __graft_entry__.build() "
                             "(or python -m paper_2508_09035_amd.build)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    dp = ctypes.POINTER(AttnDesc)
    lib.pdd_prefill_attn.restype = ctypes.c_int
    lib.pdd_prefill_attn.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.pdd_prefill_attn_chunked.restype = ctypes.c_int
    lib.pdd_prefill_attn_chunked.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.pdd_prefill_attn_chunked_noalloc.restype = ctypes.c_int
    lib.pdd_prefill_attn_chunked_noalloc.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
    lib.pdd_token_importance.restype = ctypes.c_int
    lib.pdd_token_importance.argtypes = [dp, vp, vp, vp, vp, vp, sz, vp]
    lib.pdd_select_topk.restype = ctypes.c_int
    lib.pdd_select_topk.argtypes = [vp, i32, i32, i32, vp, vp, i32, vp, vp, vp, vp, i32, vp, vp,
                                    vp, sz, vp]
    lib.pdd_select_topk_pooled.restype = ctypes.c_int
    lib.pdd_select_topk_pooled.argtypes = [vp, i32, i32, i32, vp, vp, i32, vp, vp, vp, vp, i32, i32,
                                           i32, vp, vp, vp, vp, sz, vp]
    lib.pdd_select_sentences.restype = ctypes.c_int
    lib.pdd_select_sentences.argtypes = [vp, i32, i32, i32, vp, vp, i32, vp, vp, i32, i32, vp, vp,
                                         i32, vp, vp, vp, vp, vp]
    lib.pdd_aggregate_scores.restype = ctypes.c_int
    lib.pdd_aggregate_scores.argtypes = [vp, i32, i32, i32, ctypes.c_int64, vp, i32, i32, vp, vp]
    lib.pdd_choose_r_L.restype = ctypes.c_int
    lib.pdd_choose_r_L.argtypes = [ctypes.POINTER(RLModel), i32, ctypes.POINTER(ctypes.c_double),
                                   ctypes.POINTER(ctypes.c_int32)]
    lib.pdd_pack_mask_layout.restype = ctypes.c_int64
    lib.pdd_pack_mask_layout.argtypes = [i32, vp, vp]
    lib.pdd_pack_mask.restype = ctypes.c_int
    lib.pdd_pack_mask.argtypes = [vp, i32, i32, i32, vp, vp, i32, vp, i32, vp, vp]
    lib.pdd_workspace_bytes.restype = sz
    lib.pdd_workspace_bytes.argtypes = [dp, ctypes.c_int]
    lib.pdd_last_error.restype = ctypes.c_char_p
    lib.pdd_version.restype = ctypes.c_char_p
    lib.pdd_set_option.restype = ctypes.c_int
    lib.pdd_set_option.argtypes = [ctypes.c_int, ctypes.c_int]
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        raise PddError(status, load_library().pdd_last_error().decode())


def version() -> str:
    return load_library().pdd_version().decode()


def set_option(option: int, value: int) -> None:
    _check(load_library().pdd_set_option(option, value))


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> Optional[int]:
    import torch
    return torch.cuda.current_stream().cuda_stream or None


def _host_i32(a):
    """Keep a contiguous int32 host array alive and return (array, address)."""
    import numpy as np
    if a is None:
        return None, None
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data


def make_desc(q, k, v, o, cu_seqlens_q, cu_seqlens_k, max_seqlen_q: int, max_seqlen_k: int,
              softmax_scale: float = 0.0, window: int = 0, cu_seqlens_q_host=None,
              cu_seqlens_k_host=None):
    """Fill a descriptor from [total, heads, d] tensors (v / o may be None for
    the importance-only call).  Returns (desc, keepalive)."""
    qh, qh_addr = _host_i32(cu_seqlens_q_host)
    kh, kh_addr = _host_i32(cu_seqlens_k_host)
    d = AttnDesc()
    d.batch = cu_seqlens_q.numel() - 1
    d.n_q_heads, d.n_kv_heads, d.head_dim = q.shape[1], k.shape[1], q.shape[2]
    d.total_q, d.total_k = q.shape[0], k.shape[0]
    d.max_seqlen_q, d.max_seqlen_k = int(max_seqlen_q), int(max_seqlen_k)
    d.cu_seqlens_q, d.cu_seqlens_k = cu_seqlens_q.data_ptr(), cu_seqlens_k.data_ptr()
    d.cu_seqlens_q_host, d.cu_seqlens_k_host = qh_addr, kh_addr
    d.q_stride_tok, d.q_stride_head = q.stride(0), q.stride(1)
    d.k_stride_tok, d.k_stride_head = k.stride(0), k.stride(1)
    if v is not None:
        d.v_stride_tok, d.v_stride_head = v.stride(0), v.stride(1)
    if o is not None:
        d.o_stride_tok, d.o_stride_head = o.stride(0), o.stride(1)
    d.softmax_scale = float(softmax_scale)
    d.window = int(window)
    return d, (qh, kh)


def workspace_bytes(desc: AttnDesc, which_call: int) -> int:
    return int(load_library().pdd_workspace_bytes(ctypes.byref(desc), which_call))


def _check_tensors(*ts):
    for t in ts:
        if t is not None and (not t.is_cuda or t.stride(-1) != 1):
            raise ValueError("tensors must live on the GPU with a contiguous last axis")


def prefill_attn(q, k, v, o, lse, importance, cu_seqlens_q, cu_seqlens_k, max_seqlen_q,
                 max_seqlen_k, softmax_scale=0.0, window=0, cu_seqlens_q_host=None,
                 cu_seqlens_k_host=None, workspace=None):
    """pdd_prefill_attn: writes o (bf16), lse (fp32 [Hq,total_q]) and, when
    window > 0, importance (fp32 [Hkv,total_k])."""
    _check_tensors(q, k, v, o, lse, importance)
    desc, keep = make_desc(q, k, v, o, cu_seqlens_q, cu_seqlens_k, max_seqlen_q, max_seqlen_k,
                           softmax_scale, window, cu_seqlens_q_host, cu_seqlens_k_host)
    _check(load_library().pdd_prefill_attn(
        ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(importance),
        _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
        _stream()))
    del keep


def prefill_attn_chunked(q_chunk, k_all, v_all, o, lse, importance, cu_seqlens_q, cu_seqlens_k,
                         max_seqlen_q, max_seqlen_k, softmax_scale=0.0, cu_seqlens_q_host=None,
                         cu_seqlens_k_host=None, workspace=None):
    """pdd_prefill_attn_chunked: new query chunk vs KV prefix + chunk."""
    _check_tensors(q_chunk, k_all, v_all, o, lse, importance)
    desc, keep = make_desc(q_chunk, k_all, v_all, o, cu_seqlens_q, cu_seqlens_k, max_seqlen_q,
                           max_seqlen_k, softmax_scale, 0, cu_seqlens_q_host, cu_seqlens_k_host)
    _check(load_library().pdd_prefill_attn_chunked(
        ctypes.byref(desc), _ptr(q_chunk), _ptr(k_all), _ptr(v_all), _ptr(o), _ptr(lse),
        _ptr(importance), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))
    del keep


def prefill_attn_chunked_noalloc(q_chunk, k_all, v_all, o, lse, importance, cu_seqlens_q, cu_seqlens_k,
                                 max_seqlen_q, max_seqlen_k, softmax_scale=0.0, cu_seqlens_q_host=None,
                                 cu_seqlens_k_host=None):
    """pdd_prefill_attn_chunked_noalloc: the chunked call on the library's built-in scratch."""
    _check_tensors(q_chunk, k_all, v_all, o, lse, importance)
    desc, keep = make_desc(q_chunk, k_all, v_all, o, cu_seqlens_q, cu_seqlens_k, max_seqlen_q,
                           max_seqlen_k, softmax_scale, 0, cu_seqlens_q_host, cu_seqlens_k_host)
    _check(load_library().pdd_prefill_attn_chunked_noalloc(
        ctypes.byref(desc), _ptr(q_chunk), _ptr(k_all), _ptr(v_all), _ptr(o), _ptr(lse),
        _ptr(importance), _stream()))
    del keep


def token_importance(q, k, lse, importance, cu_seqlens_q, cu_seqlens_k, max_seqlen_q,
                     max_seqlen_k, softmax_scale=0.0, window=-1, cu_seqlens_q_host=None,
                     cu_seqlens_k_host=None, workspace=None):
    """pdd_token_importance: importance from precomputed lse."""
    _check_tensors(q, k, lse, importance)
    desc, keep = make_desc(q, k, None, None, cu_seqlens_q, cu_seqlens_k, max_seqlen_q,
                           max_seqlen_k, softmax_scale, window, cu_seqlens_q_host,
                           cu_seqlens_k_host)
    _check(load_library().pdd_token_importance(
        ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(lse), _ptr(importance), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))
    del keep


def select_topk(scores, cu_seqlens_k, max_seqlen_k, k_per_seq, cu_keep, total_keep, out_indices,
                out_mask=None, cand_begin=None, cand_end=None, cu_seqlens_k_host=None,
                workspace=None):
    """pdd_select_topk: scores fp32 [n_heads,total_k] -> ascending kept indices
    int32 [n_heads,total_keep] and optional uint8 mask [n_heads,total_k]."""
    _check_tensors(scores, out_indices, out_mask)
    kh, kh_addr = _host_i32(cu_seqlens_k_host)
    _check(load_library().pdd_select_topk(
        _ptr(scores), scores.shape[0], cu_seqlens_k.numel() - 1, scores.shape[1],
        _ptr(cu_seqlens_k), kh_addr, int(max_seqlen_k), _ptr(cand_begin), _ptr(cand_end),
        _ptr(k_per_seq), _ptr(cu_keep), int(total_keep), _ptr(out_indices), _ptr(out_mask),
        _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
        _stream()))
    del kh


POOL_NONE, POOL_MAX, POOL_AVG = 0, 1, 2


def select_topk_pooled(scores, cu_seqlens_k, max_seqlen_k, k_per_seq, cu_keep, total_keep,
                       out_indices, out_mask=None, pool_kernel=1, pool_mode=POOL_NONE,
                       pooled_out=None, cand_begin=None, cand_end=None, cu_seqlens_k_host=None):
    """pdd_select_topk_pooled: 1-D pooling (max / zero-padded average, odd kernel) of the scores
    along each sequence, then the same selection as select_topk."""
    _check_tensors(scores, out_indices, out_mask, pooled_out)
    kh, kh_addr = _host_i32(cu_seqlens_k_host)
    _check(load_library().pdd_select_topk_pooled(
        _ptr(scores), scores.shape[0], cu_seqlens_k.numel() - 1, scores.shape[1],
        _ptr(cu_seqlens_k), kh_addr, int(max_seqlen_k), _ptr(cand_begin), _ptr(cand_end),
        _ptr(k_per_seq), _ptr(cu_keep), int(total_keep), int(pool_kernel), int(pool_mode),
        _ptr(pooled_out), _ptr(out_indices), _ptr(out_mask), None, 0, _stream()))
    del kh


SENT_SUM, SENT_MEAN = 0, 1


def select_sentences(scores, cu_seqlens_k, max_seqlen_k, cu_sent, sent_end, max_sent_per_seq,
                     token_budget, agg_mode=SENT_MEAN, cand_begin=None, out_sent_scores=None,
                     out_sent_keep=None, out_mask=None, out_kept_tokens=None,
                     cu_seqlens_k_host=None):
    """pdd_select_sentences: rank sentences by summed / mean token score, keep the longest
    prefix of the ranking that fits the token budget."""
    _check_tensors(scores, out_sent_scores, out_sent_keep, out_mask)
    kh, kh_addr = _host_i32(cu_seqlens_k_host)
    _check(load_library().pdd_select_sentences(
        _ptr(scores), scores.shape[0], cu_seqlens_k.numel() - 1, scores.shape[1],
        _ptr(cu_seqlens_k), kh_addr, int(max_seqlen_k), _ptr(cu_sent), _ptr(sent_end),
        sent_end.numel(), int(max_sent_per_seq), _ptr(cand_begin), _ptr(token_budget),
        int(agg_mode), _ptr(out_sent_scores), _ptr(out_sent_keep), _ptr(out_mask),
        _ptr(out_kept_tokens), _stream()))
    del kh


def aggregate_scores(scores, out, layer_weights=None, reduce_heads=False, accumulate=False):
    """pdd_aggregate_scores: scores fp32 [n_layers, n_heads, total_k] (layers may be strided)
    -> out fp32 [n_heads or 1, total_k], weighted sum over layers (and heads)."""
    _check_tensors(scores, out, layer_weights)
    if scores.dim() != 3 or scores.stride(2) != 1 or scores.stride(1) != scores.shape[2]:
        raise ValueError("scores must be [n_layers, n_heads, total_k] with contiguous layers")
    _check(load_library().pdd_aggregate_scores(
        _ptr(scores), scores.shape[0], scores.shape[1], scores.shape[2], scores.stride(0),
        _ptr(layer_weights), int(bool(reduce_heads)), int(bool(accumulate)), _ptr(out), _stream()))


def choose_r_L(l, k_c, k_d, delta, xi_scene, tpot_c, tpot_d, tau, delta_cloud=0.0):
    """pdd_choose_r_L (host only): closed-form (r, L) of the paper's program P; raises PddError
    when the constraints admit no solution."""
    m = RLModel(k_c, k_d, delta, xi_scene, tpot_c, tpot_d, tau, delta_cloud)
    r, L = ctypes.c_double(), ctypes.c_int32()
    _check(load_library().pdd_choose_r_L(ctypes.byref(m), int(l), ctypes.byref(r), ctypes.byref(L)))
    return r.value, L.value


def pack_mask_layout(cu_seqlens_k_host):
    """pdd_pack_mask_layout (host only): int32 numpy prefix sums of the per-sequence byte
    counts of the bit stream, and the bytes per row."""
    import numpy as np
    cu = np.ascontiguousarray(cu_seqlens_k_host, dtype=np.int32)
    out = np.zeros(len(cu), dtype=np.int32)
    total = load_library().pdd_pack_mask_layout(len(cu) - 1, cu.ctypes.data, out.ctypes.data)
    if total < 0:
        raise PddError(-1, load_library().pdd_last_error().decode())
    return out, int(total)


def pack_mask(mask, cu_seqlens_k, max_seqlen_k, cu_bytes, total_bytes, out_bits,
              cu_seqlens_k_host=None):
    """pdd_pack_mask: uint8 mask [rows,total_k] -> bit stream [rows,total_bytes], per sequence
    byte-aligned, first token in the most significant bit."""
    _check_tensors(mask, out_bits)
    kh, kh_addr = _host_i32(cu_seqlens_k_host)
    _check(load_library().pdd_pack_mask(
        _ptr(mask), mask.shape[0], cu_seqlens_k.numel() - 1, mask.shape[1], _ptr(cu_seqlens_k),
        kh_addr, int(max_seqlen_k), _ptr(cu_bytes), int(total_bytes), _ptr(out_bits), _stream()))
    del kh
