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
  O5  the appendix speaks of shots and of mandatory elements such as the global
      caption; here every caption span is a (mandatory) segment of its own and
      the video chunks of a shot form one competing segment (`segments`); the
      reduced stream keeps each kept token's chunk, shot, window and caption
      membership (`reduce_layout`).
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


def segments(offsets: Sequence[int], shot: Sequence[int], text_spans) -> tuple:
    """The segments the outer router sees (reading O5): the stream is cut wherever a caption span
    starts or ends and wherever the shot id changes; a caption span is a segment of its own, the
    video chunks of a shot between two captions form one segment.
    -> (seg_offsets [P+1], is_caption [P])."""
    off = [int(t) for t in offsets]
    spans = [(int(a), int(b)) for a, b in np.asarray(text_spans).reshape(-1, 2)]
    cuts = {off[0], off[-1]}
    for a, b in spans:
        cuts.update((a, b))
    for j in range(1, len(off) - 1):
        if shot[j] != shot[j - 1]:
            cuts.add(off[j])
    seg = sorted(cuts)
    cap = [int(any(a <= seg[p] and seg[p + 1] <= b for a, b in spans)) for p in range(len(seg) - 1)]
    return np.asarray(seg, dtype=np.int64), np.asarray(cap, dtype=np.int64)


def reduce_layout(offsets, shot, window, text_spans, seg_off, kept):
    """Layout of the reduced stream (reading O3: kept segments in stream order): token by token,
    every kept token keeps its chunk, its chunk's shot and window ids and its caption flag; chunk
    boundaries, and caption spans, of the reduced stream are where those change or where a kept
    segment ends. -> dict(offsets, shot, window, text_spans)."""
    off = np.asarray(offsets, dtype=np.int64)
    N, C = int(off[-1]), len(off) - 1
    chunk_of = np.zeros(N, dtype=np.int64)
    for j in range(C):
        chunk_of[off[j]:off[j + 1]] = j
    in_span = np.full(N, -1, dtype=np.int64)
    for s, (a, b) in enumerate(np.asarray(text_spans).reshape(-1, 2)):
        in_span[a:b] = s
    win = np.arange(C) if window is None else np.asarray(window)
    new_off, new_shot, new_win, new_spans = [0], [], [], []
    pos = 0
    for sg in kept:
        rows = np.arange(seg_off[sg], seg_off[sg + 1])
        if len(rows) == 0:
            raise ValueError("empty segment")
        first, last = chunk_of[rows[0]], chunk_of[rows[-1]]
        if rows[0] != off[first] or rows[-1] + 1 != off[last + 1]:
            raise ValueError("segment boundaries must be chunk boundaries")
        span_start = None
        for t, r in enumerate(rows):
            if t == 0 or chunk_of[r] != chunk_of[r - 1]:                  # a chunk begins
                if t > 0:
                    new_off.append(pos + t)
                new_shot.append(int(shot[chunk_of[r]]))
                new_win.append(int(win[chunk_of[r]]))
            if in_span[r] >= 0 and (t == 0 or in_span[r - 1] != in_span[r]):
                span_start = pos + t
            if in_span[r] >= 0 and (t == len(rows) - 1 or in_span[r + 1] != in_span[r]):
                new_spans.append((span_start, pos + t + 1))
        pos += len(rows)
        new_off.append(pos)
    return dict(offsets=np.asarray(new_off, dtype=np.int32), shot=np.asarray(new_shot, dtype=np.int32),
                window=np.asarray(new_win, dtype=np.int32),
                text_spans=np.asarray(new_spans, dtype=np.int32).reshape(-1, 2))
