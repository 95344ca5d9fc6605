"""CPU oracle for the prefill-attention + prompt-refinement path.

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports it and it
never imports the product package.

* `attention`, `importance` call the plain fp64 C definition in
  `pdd_oracle.c` (Section 2.2.3 attention equation; Section 3.2 "Prompt
  Refiner": window weights summed along the query dimension).
* `select_topk` is the refiner's selection step written as a full sort
  (Section 3.2: sort the summed scores, keep the top values at ratio r, filter
  the positions; Section 3.2 mask tensor: 1 at position i = token i selected).
"""
from .core import (
    build,
    attention,
    importance,
    select_topk,
    pack_mask,
    pool_scores,
    select_sentences,
    aggregate_scores,
    choose_r_L,
    num_threads,
    widen_bf16,
)

__all__ = ["build", "attention", "importance", "select_topk", "pack_mask", "pool_scores", "select_sentences", "aggregate_scores", "choose_r_L", "num_threads", "widen_bf16"]
