"""CPU oracle of the outer-loop context routing (App. "Outer Loop Context Routing").

TEST INFRASTRUCTURE ONLY: imported by tests/ and the benchmark's cpu-baseline
leg. Plain numpy in float64; nothing here is shared with the HIP path.

The appendix fixes: the token stream is partitioned into P large segments
(e.g. shots); each segment's descriptor is the mean of its token features; the
current block g is summarised by its own mean; the score of segment j is the
inner product of the two; the M best-scoring segments are kept and concatenated
with the mandatory elements to form the reduced stream handed to the inner
layer. Readings where it is silent:

  O1  the candidates are the segments other than g that are not mandatory, and,
      with `causal`, only those before g (the history of an autoregressive
      roll-out);
  O2  fewer than M candidates: all of them are kept; ties go to the lower index;
  O3  the reduced stream keeps the original order of the stream: mandatory
      segments, selected segments and g itself, ascending by position;
  O4  features enter as stored (bf16 or fp32 values), means and scores are exact
      here; the product accumulates in fp32.
"""
from __future__ import annotations

from typing import Optional, Sequence

import numpy as np


def segment_means(x: np.ndarray, seg_off: Sequence[int]) -> np.ndarray:
    """x [N, D] -> [P, D]: arithmetic mean of the rows of each segment."""
    x = np.asarray(x, dtype=np.float64)
    return np.stack([x[seg_off[j]:seg_off[j + 1]].mean(axis=0) for j in range(len(seg_off) - 1)])


def outer_route(x: np.ndarray, seg_off: Sequence[int], mandatory: Optional[Sequence[int]], g: int, M: int,
                causal: bool = True):
    """-> selected [M] (best first, -1 padded), scores [P] (inner products with segment g's mean),
    kept (ascending list of the segments of the reduced stream), means [P, D]."""
    P = len(seg_off) - 1
    mand = np.zeros(P, bool) if mandatory is None else np.asarray(mandatory).astype(bool)
    means = segment_means(x, seg_off)
    scores = means @ means[g]
    cand = [j for j in range(P) if j != g and not mand[j] and (not causal or j < g)]
    best = sorted(cand, key=lambda j: (-scores[j], j))[:max(M, 0)]
    selected = np.full(max(M, 0), -1, dtype=np.int32)
    selected[:len(best)] = best
    kept = sorted(set(best) | set(np.nonzero(mand)[0].tolist()) | {g})
    return selected, scores, kept, means


def reduced_rows(seg_off: Sequence[int], kept: Sequence[int]) -> np.ndarray:
    """Source row of every row of the reduced stream (O3)."""
    parts = [np.arange(seg_off[j], seg_off[j + 1]) for j in kept]
    return np.concatenate(parts) if parts else np.zeros(0, dtype=np.int64)
