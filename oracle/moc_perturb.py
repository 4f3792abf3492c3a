"""CPU oracle of the routing regularisers: context drop-off and context drop-in
(Sec. 3.2, "Context Drop-off" and "Context Drop-in").

TEST INFRASTRUCTURE ONLY: imported by tests/. Plain Python over numpy arrays,
one query at a time; nothing here is shared with the HIP path.

What the paper fixes: after routing, per query, a drop probability
p ~ Uniform(0, p_max) is drawn and floor(p * k) randomly chosen chunks are
removed from the routed set; independently m ~ Poisson(lambda) randomly chosen
chunks are added to it. What it leaves open, and the reading taken here:

  R1  "per query" is per (batch, head, query): routing is per head.
  R2  the random numbers come from Philox4x32-10 (Salmon et al., SC'11), one
      stream per (batch*H + head, query): counter (query, batch*H + head, block, 0),
      key (seed low word, seed high word); draw t is word t mod 4 of block t / 4.
      Draw 0 gives p, draw 1 gives m, the following draws pick the chunks to
      remove, then the chunks to add.
  R3  p = u * p_max with u = (draw >> 8) * 2^-24; the count floor(p * k) uses the
      layer's k (not the number of chunks actually routed) and is evaluated in
      single precision, (u * p_max) * k, because it decides an integer; it is
      capped by the number of routed chunks of the query.
  R4  removal is uniform without replacement: each pick takes entry
      floor(draw * n / 2^32) of the n entries still alive, in their routed order.
      Survivors keep their order (best first).
  R5  m = #{ j < max_in : draw >= floor(CDF_lambda(j) * 2^32) }, i.e. Poisson by
      inversion, truncated at max_in (the output has a fixed width), and capped
      by the number of chunks available.
  R6  the chunks added are drawn uniformly without replacement from the
      query's routing candidates (same eligibility as routing: not a forced
      link, earlier than the query's chunk under the causal mask) that were not
      routed for this query - a chunk removed by drop-off does not come back.
      Each pick takes entry floor(draw * n / 2^32) of the n available chunks in
      ascending index order.
  R7  output row, width k + max_in: survivors, then added chunks in draw order,
      then -1.
"""
from __future__ import annotations

import math
from typing import Optional, Sequence

import numpy as np

_M0, _M1 = 0xD2511F53, 0xCD9E8D57
_W0, _W1 = 0x9E3779B9, 0xBB67AE85
_MASK = 0xFFFFFFFF


def philox4x32_10(counter, key):
    """One block of Philox4x32 with 10 rounds: 4 counter words, 2 key words -> 4 words."""
    c0, c1, c2, c3 = (int(x) & _MASK for x in counter)
    k0, k1 = (int(x) & _MASK for x in key)
    for _ in range(10):
        p0 = _M0 * c0
        p1 = _M1 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & _MASK, p1 & _MASK, ((p0 >> 32) ^ c3 ^ k1) & _MASK, p0 & _MASK
        k0 = (k0 + _W0) & _MASK
        k1 = (k1 + _W1) & _MASK
    return c0, c1, c2, c3


class Draws:
    """The stream of one (bh, query): draw t = word t mod 4 of block t / 4 (R2)."""

    def __init__(self, seed: int, bh: int, i: int):
        self.key = (seed & _MASK, (seed >> 32) & _MASK)
        self.bh, self.i, self.t, self.block = bh, i, 0, None

    def next(self) -> int:
        blk, w = divmod(self.t, 4)
        if w == 0 or self.block is None:
            self.block = philox4x32_10((self.i, self.bh, blk, 0), self.key)
        self.t += 1
        return self.block[w]


def poisson_thresholds(lam: float, max_in: int):
    """floor(CDF_lambda(j) * 2^32) for j < max_in, by the recurrence pmf(j) = pmf(j-1) * lambda / j (R5)."""
    out, term, cdf = [], math.exp(-lam), 0.0
    for j in range(max_in):
        if j > 0:
            term = term * lam / j
        cdf += term
        out.append(int(math.floor(min(cdf, 1.0) * 4294967296.0)))
    return out


def n_drop(draw: int, p_max: float, k: int) -> int:
    """floor(p * k), p = u * p_max, in single precision (R3)."""
    u = np.float32(draw >> 8) * np.float32(2.0 ** -24)
    p = np.float32(u * np.float32(p_max))
    return int(math.floor(float(np.float32(p * np.float32(k)))))


def perturb_row(row: Sequence[int], candidates: Sequence[int], k: int, p_max: float, thresholds: Sequence[int],
                max_in: int, draws: Draws):
    """row: routed chunks of one query (best first, -1 padded); candidates: its eligible chunks, ascending."""
    routed = [int(c) for c in row if c >= 0]
    r_drop, r_in = draws.next(), draws.next()
    # drop-off (R3, R4)
    alive = list(range(len(routed)))
    for _ in range(min(n_drop(r_drop, p_max, k), len(routed))):
        alive.pop((draws.next() * len(alive)) >> 32)
    kept = [routed[a] for a in alive]
    # drop-in (R5, R6)
    avail = [int(c) for c in candidates if int(c) not in routed]
    m = sum(1 for t in thresholds[:max_in] if r_in >= t)
    added = []
    for _ in range(min(m, len(avail))):
        added.append(avail.pop((draws.next() * len(avail)) >> 32))
    out = kept + added
    return out + [-1] * (k + max_in - len(out))


def candidates_of(L, i: int, causal: bool):
    """Routing candidates of query i: chunks that are not forced links (Sec. 3.3: captions, own
    window) and, under the causal mask (Sec. 3.2), lie before the query's chunk."""
    cq = int(L.chunk_of[i])
    hi = cq if causal else L.C
    return [j for j in range(hi) if L.kind[j] == 0 and L.win[j] != L.win[cq]]


def perturb(L, sel: np.ndarray, topk: int, causal: bool, p_max: float, lam: float, max_in: int, seed: int,
            qidx: Optional[Sequence[int]] = None, heads: Optional[Sequence[int]] = None, H: Optional[int] = None):
    """sel [B,Hs,nq,topk] (rows of queries qidx, default all N) -> [B,Hs,nq,topk+max_in].

    heads: the head index of each slice of sel's second axis within a layer of H heads
    (default: sel holds all H heads)."""
    B, Hs, nq, _ = sel.shape
    qi = np.arange(L.N) if qidx is None else np.asarray(qidx)
    heads = list(range(Hs)) if heads is None else list(heads)
    H = Hs if H is None else H
    thr = poisson_thresholds(lam, max_in)
    out = np.full((B, Hs, nq, topk + max_in), -1, dtype=np.int32)
    cand_cache = {}
    for r, i in enumerate(qi):
        cq = int(L.chunk_of[i])
        if cq not in cand_cache:
            cand_cache[cq] = candidates_of(L, int(i), causal)
        for b in range(B):
            for hs, h in enumerate(heads):
                out[b, hs, r] = perturb_row(sel[b, hs, r], cand_cache[cq], topk, p_max, thr, max_in,
                                            Draws(seed, b * H + h, int(i)))
    return out
