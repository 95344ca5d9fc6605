"""Input recipes.

Every tensor is drawn as float32 from ``numpy.random.default_rng(seed)``
(PCG64) in the fixed order Q, K, V, multiplied by the recipe's gain, rounded
to bf16 with round-to-nearest-even and stored as the raw 16-bit pattern.
Nothing here evaluates the method; `keep_count` is the only arithmetic and it
is the caller-side choice of k from a keep ratio (refinement ratio r =
refined length / original length, Section 2.2.3 "Analysis on Assistance").
"""
from __future__ import annotations

from dataclasses import dataclass, field
from fractions import Fraction
from typing import Optional, Sequence

import numpy as np

CONFIG_NAMES = ("c1", "c2", "c3", "c4", "c5", "c4h")

# Lengths of the eight packed prompts of the ragged workload.  They were drawn
# once with `c3_lengths_from_recipe()` and are frozen here so that every
# consumer shares the same integers (a test re-derives them).
C3_LENGTHS = (2360, 1384, 1502, 512, 7898, 4831, 1604, 3659)


def c3_lengths_from_recipe(seed: int = 2, n: int = 8, median: int = 2048,
                           sigma: float = 0.75, lo: int = 512, hi: int = 8192):
    """len_b = clip(round(exp(ln median + sigma * z_b)), lo, hi), z ~ N(0,1)."""
    z = np.random.default_rng(seed).standard_normal(n)
    return tuple(int(x) for x in
                 np.clip(np.rint(np.exp(np.log(median) + sigma * z)), lo, hi))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even); returns uint16 patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32)
            << np.uint32(16)).view(np.float32)


def keep_count(n_candidates: int, ratio) -> int:
    """k = max(1, floor(r * n)) with r an exact rational (e.g. "3/10", 0.25)."""
    r = Fraction(str(ratio)) if not isinstance(ratio, Fraction) else ratio
    if n_candidates <= 0:
        return 0
    return max(1, (r.numerator * n_candidates) // r.denominator)


@dataclass
class Workload:
    """One packed batch.  q: [total_q, Hq, d], k/v: [total_k, Hkv, d], uint16
    bf16 patterns; cu_seqlens_*: int32 [B+1]; window W (0 = no importance);
    cand_begin/cand_end: candidate key range per sequence (sequence-local);
    k_keep: per-sequence number of indices to select per KV head."""
    name: str
    q: np.ndarray
    k: np.ndarray
    v: np.ndarray
    cu_seqlens_q: np.ndarray
    cu_seqlens_k: np.ndarray
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    window: int
    chunked: bool
    scale: float
    keep_ratio: Fraction
    cand_begin: np.ndarray
    cand_end: np.ndarray
    k_keep: np.ndarray
    seed: int
    notes: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def batch(self) -> int:
        return len(self.cu_seqlens_q) - 1

    @property
    def total_q(self) -> int:
        return int(self.cu_seqlens_q[-1])

    @property
    def total_k(self) -> int:
        return int(self.cu_seqlens_k[-1])

    @property
    def seqlens_q(self) -> np.ndarray:
        return np.diff(self.cu_seqlens_q)

    @property
    def seqlens_k(self) -> np.ndarray:
        return np.diff(self.cu_seqlens_k)

    @property
    def cu_keep(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.k_keep)]).astype(np.int32)

    def causal_pairs(self) -> int:
        """Number of (query, key) pairs under the bottom-right aligned causal
        mask, summed over sequences (one head)."""
        nq = self.seqlens_q.astype(np.int64)
        nk = self.seqlens_k.astype(np.int64)
        return int(np.sum(nq * (nk - nq) + nq * (nq + 1) // 2))

    def window_pairs(self) -> int:
        """Pairs visited by the observation-window rows (one head)."""
        if self.window <= 0 and not self.chunked:
            return 0
        nq = self.seqlens_q.astype(np.int64)
        nk = self.seqlens_k.astype(np.int64)
        w = nq if self.chunked else np.minimum(self.window, nq)
        # rows nq-w .. nq-1 ; row i sees i + (nk-nq) + 1 keys
        first = nq - w + (nk - nq) + 1
        last = nk
        return int(np.sum(w * (first + last) // 2))

    def attn_flops(self) -> int:
        return 4 * self.head_dim * self.n_q_heads * self.causal_pairs()

    def importance_flops(self) -> int:
        return 2 * self.head_dim * self.n_q_heads * self.window_pairs()


def _draw(rng, shape, gain):
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if gain != 1.0:
        x *= np.float32(gain)
    return x


def _cu(lengths: Sequence[int]) -> np.ndarray:
    return np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)


def make_custom(name: str, seqlens_q: Sequence[int], seqlens_k: Optional[Sequence[int]],
                n_q_heads: int, n_kv_heads: int, head_dim: int, window: int,
                keep_ratio="1/2", seed: int = 0, gain: float = 1.0,
                chunked: bool = False, scale: Optional[float] = None,
                notes: str = "") -> Workload:
    """General recipe used by the named configs and by edge-case tests."""
    seqlens_q = [int(x) for x in seqlens_q]
    seqlens_k = seqlens_q if seqlens_k is None else [int(x) for x in seqlens_k]
    assert len(seqlens_q) == len(seqlens_k)
    rng = np.random.default_rng(seed)
    tq, tk = sum(seqlens_q), sum(seqlens_k)
    q = _draw(rng, (tq, n_q_heads, head_dim), gain)
    k = _draw(rng, (tk, n_kv_heads, head_dim), gain)
    v = _draw(rng, (tk, n_kv_heads, head_dim), gain)
    ratio = Fraction(str(keep_ratio))
    if chunked:
        # candidates are the existing prefix only; the chunk's own keys are kept
        cand_begin = np.zeros(len(seqlens_q), dtype=np.int32)
        cand_end = np.array([nk - nq for nq, nk in zip(seqlens_q, seqlens_k)], dtype=np.int32)
    else:
        cand_begin = np.zeros(len(seqlens_q), dtype=np.int32)
        cand_end = np.array(seqlens_k, dtype=np.int32)
    k_keep = np.array([keep_count(int(e - b), ratio) for b, e in zip(cand_begin, cand_end)],
                      dtype=np.int32)
    return Workload(
        name=name, q=f32_to_bf16_bits(q), k=f32_to_bf16_bits(k), v=f32_to_bf16_bits(v),
        cu_seqlens_q=_cu(seqlens_q), cu_seqlens_k=_cu(seqlens_k),
        n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, head_dim=head_dim,
        window=window, chunked=chunked,
        scale=float(scale) if scale is not None else 1.0 / float(np.sqrt(head_dim)),
        keep_ratio=ratio, cand_begin=cand_begin, cand_end=cand_end, k_keep=k_keep,
        seed=seed, notes=notes)


def _heavy_hitter(name: str, n: int, seed: int, boost_window_queries: bool) -> Workload:
    """Long prompt with 1% of key positions shifted by +3 along one random unit
    direction per KV head (a few keys draw most of the attention mass, as in
    the attention-weight distributions of Section 4.4).  With
    `boost_window_queries` the last W queries are also shifted by sqrt(d)
    along that direction so that the marked keys gain about +3 logits."""
    hq, hkv, d, w = 32, 8, 128, 128
    rng = np.random.default_rng(seed)
    q = _draw(rng, (n, hq, d), 1.0)
    k = _draw(rng, (n, hkv, d), 1.0)
    v = _draw(rng, (n, hkv, d), 1.0)
    n_heavy = int(round(0.01 * n))
    heavy = np.zeros((hkv, n_heavy), dtype=np.int64)
    for g in range(hkv):
        u = rng.standard_normal(d).astype(np.float32)
        u /= np.float32(np.linalg.norm(u))
        pos = np.sort(rng.choice(n, size=n_heavy, replace=False))
        heavy[g] = pos
        k[pos, g, :] += np.float32(3.0) * u
        if boost_window_queries:
            grp = hq // hkv
            q[n - w:, g * grp:(g + 1) * grp, :] += np.float32(np.sqrt(d)) * u
    ratio = Fraction(1, 10)
    return Workload(
        name=name, q=f32_to_bf16_bits(q), k=f32_to_bf16_bits(k), v=f32_to_bf16_bits(v),
        cu_seqlens_q=_cu([n]), cu_seqlens_k=_cu([n]),
        n_q_heads=hq, n_kv_heads=hkv, head_dim=d, window=w, chunked=False,
        scale=1.0 / float(np.sqrt(d)), keep_ratio=ratio,
        cand_begin=np.zeros(1, np.int32), cand_end=np.array([n], np.int32),
        k_keep=np.array([keep_count(n, ratio)], np.int32), seed=seed,
        notes="1% heavy-hitter keys (+3 on a random unit direction per KV head)",
        extra={"heavy_positions": heavy})


def make_workload(name: str, n_override: Optional[int] = None) -> Workload:
    """The five benchmark configurations (plus `c4h`, the boosted-query variant
    of the long prompt).  `n_override` shrinks the sequence length(s) while
    keeping heads / head_dim / window / ratio, for quick checks."""
    if name == "c1":
        n = n_override or 512
        return make_custom("c1", [n], None, 1, 1, 64, 32, "1/2", seed=0, gain=1.0,
                           notes="tiny single-head causal prefill")
    if name == "c2":
        n = n_override or 4096
        return make_custom("c2", [n], None, 32, 8, 128, 64, "3/10", seed=1, gain=0.5,
                           notes="Llama-3-8B-shaped layer, GQA 4:1")
    if name == "c3":
        lens = list(C3_LENGTHS)
        if n_override:
            lens = [max(1, (x * n_override) // 8192) for x in lens]
        return make_custom("c3", lens, None, 32, 8, 128, 64, "1/2", seed=2, gain=1.0,
                           notes="ragged packed batch, log-normal lengths")
    if name == "c4":
        return _heavy_hitter("c4", n_override or 32768, seed=3, boost_window_queries=False)
    if name == "c4h":
        return _heavy_hitter("c4h", n_override or 32768, seed=3, boost_window_queries=True)
    if name == "c5":
        prefix = n_override or 8192
        chunk = 256
        return make_custom("c5", [chunk] * 4, [prefix + chunk] * 4, 64, 8, 128, chunk, "1/4",
                           seed=4, gain=1.0, chunked=True,
                           notes="chunked catch-up: KV prefix + 256 new queries")
    raise KeyError(name)
