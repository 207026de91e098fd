"""CPU float64 oracle for the SurfaceLogicKV compression pass.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain definition of what
the HIP library computes, written from the paper (arXiv 2508.15806).  It shares
no code with the GPU path and must never be imported by the product package:
only the tests, the smoke check and the benchmark's CPU-baseline leg use it.

Modules
  compress  - Stage 2b: window scoring, softmax importance, pooling, top-k,
              gather (Eq. 2-4, Eq. 7-8, Algorithm 3), on a packed
              prefill batch and on an already compacted cache.
  budgets   - Stage 2a: per-head capacities (Eq. 6, Algorithm 2).
  behavior  - Stage 1: WO / WD / WS counting and SF / LG / INF scores
              (Algorithm 1).

Every function here is pinned by tests that do not call back into it (closed
forms, brute force on tiny inputs, library routines, hand-worked examples from
the paper's formulas).  Nothing is "parity unpinned"; the weakest pin is the
micro-aggregation of Stage-1 sums over several rows, for which the paper prints
no worked example (pinned by brute force only).
"""

from .compress import (  # noqa: F401
    bf16_bits_to_f64,
    fp8_e4m3_to_f64,
    window_importance,
    pool_1d,
    select_topk,
    compress_segment,
    compress_layer,
    recompress_layer,
    kept_count,
)
from .budgets import allocate_budgets, allocate_budgets_literal, allocate_budgets_per_query_head, fixed_from_beta  # noqa: F401
from .behavior import (row_weights, finalize_scores, harmonic, score_heads, score_heads_modes,  # noqa: F401
                       attention_rows, score_heads_from_qk)
