"""Pins of the drop-off / drop-in oracle (Sec. 3.2, "Context Drop-off", "Context Drop-in").

The generator is pinned to its published known-answer vectors; the Poisson draw
to scipy's quantile function; the two samplers to what uniform sampling without
replacement fixes (counts, membership, order, frequencies within chi-square
bounds) and to the special cases that reduce to the identity.
"""
import os

import numpy as np
import pytest
from scipy import stats

import moc_inputs as mi
from oracle import moc_oracle as mo
from oracle import moc_perturb as mp

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers():
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        assert list(mp.philox4x32_10(w[0:4], w[4:6])) == w[6:10]


def test_draw_streams_are_indexed_by_head_query_and_block():
    d = mp.Draws(seed=(7 << 32) | 5, bh=3, i=11)
    got = [d.next() for _ in range(9)]
    want = [w for blk in range(3) for w in mp.philox4x32_10((11, 3, blk, 0), (5, 7))][:9]
    assert got == want
    other = mp.Draws(seed=(7 << 32) | 5, bh=3, i=12)
    assert other.next() != got[0]


@pytest.mark.parametrize("lam", [0.0, 0.3, 1.0, 2.5])
def test_poisson_by_inversion_matches_the_quantile_function(lam):
    max_in = 12
    thr = mp.poisson_thresholds(lam, max_in)
    rng = np.random.default_rng(1)
    r = rng.integers(0, 1 << 32, size=4000, dtype=np.uint64)
    m = np.array([sum(1 for t in thr if int(x) >= t) for x in r])
    # smallest m with CDF(m) > r / 2^32; the half-step keeps clear of the (measure-zero) boundaries
    want = np.minimum(stats.poisson.ppf((r.astype(np.float64) + 0.5) / 4294967296.0, lam) if lam > 0 else 0, max_in)
    assert (m == want).all()
    if lam > 0:
        assert abs(m.mean() - lam) < 5 * np.sqrt(lam / len(r))


def test_drop_count_is_floor_p_k_in_single_precision():
    # p_max = 1, k = 8: floor(8 u) is the top three bits of the draw
    for draw in (0, 1 << 29, (1 << 32) - 1, 0x7fffffff, 0x80000000, 0xdeadbeef):
        assert mp.n_drop(draw, 1.0, 8) == draw >> 29
    assert mp.n_drop(0xffffffff, 0.0, 8) == 0
    assert mp.n_drop(0xffffffff, 0.5, 8) == 3          # p just below 0.5 -> floor(3.99..) = 3
    assert mp.n_drop(0x80000000, 0.5, 8) == 2          # p = 0.25 exactly


def _rows(n, k, p_max, lam, max_in, routed, cand, seed=3):
    thr = mp.poisson_thresholds(lam, max_in)
    return [mp.perturb_row(routed, cand, k, p_max, thr, max_in, mp.Draws(seed, 0, i)) for i in range(n)]


def test_identity_without_regularisers():
    routed, cand = [9, 4, 7, -1], list(range(12))
    for row in _rows(50, 4, 0.0, 0.0, 3, routed, cand):
        assert row == [9, 4, 7, -1, -1, -1, -1]


def test_drop_off_removes_uniformly_and_keeps_order():
    routed, k, n = [12, 3, 8, 5, 10, 1, 7, 2], 8, 6000
    rows = _rows(n, k, 1.0, 0.0, 0, routed, list(range(20)))
    kept_counts = np.zeros(k + 1)
    removed = np.zeros(k)
    for row in rows:
        kept = [c for c in row if c >= 0]
        assert kept == [c for c in routed if c in kept]          # survivors in routed order
        assert row[len(kept):] == [-1] * (k - len(kept))
        kept_counts[len(kept)] += 1
        for p, c in enumerate(routed):
            removed[p] += c not in kept
    # floor(8 u) is uniform on 0..7 -> 1..8 survivors, each with probability 1/8
    assert kept_counts[0] == 0
    assert stats.chisquare(kept_counts[1:]).pvalue > 1e-4
    # every position is removed equally often
    assert stats.chisquare(removed).pvalue > 1e-4


def test_drop_off_is_capped_by_the_routed_count():
    rows = _rows(400, 8, 1.0, 0.0, 0, [6, 2, -1, -1, -1, -1, -1, -1], list(range(9)))
    assert min(sum(c >= 0 for c in r) for r in rows) == 0 and max(sum(c >= 0 for c in r) for r in rows) == 2


def test_drop_in_adds_distinct_unrouted_candidates_uniformly():
    routed, cand, k, max_in, n = [5, 11, -1], [1, 2, 5, 6, 8, 11, 13, 14], 3, 4, 6000
    rows = _rows(n, k, 0.0, 1.5, max_in, routed, cand)
    avail = [c for c in cand if c not in (5, 11)]
    hits = {c: 0 for c in avail}
    m_counts = np.zeros(max_in + 1)
    for row in rows:
        assert row[:2] == [5, 11]
        added = [c for c in row[2:] if c >= 0]
        assert row[2 + len(added):] == [-1] * (k + max_in - 2 - len(added))
        assert len(set(added)) == len(added) and set(added) <= set(avail)
        m_counts[len(added)] += 1
        for c in added:
            hits[c] += 1
    pm = stats.poisson.pmf(np.arange(max_in), 1.5)
    expect = np.append(pm, 1 - pm.sum()) * n                      # truncated at max_in
    assert stats.chisquare(m_counts, expect).pvalue > 1e-4
    assert stats.chisquare(list(hits.values())).pvalue > 1e-4    # every available chunk equally often


def test_drop_in_takes_everything_when_too_few_are_available():
    rows = _rows(300, 2, 0.0, 6.0, 5, [4, 0], [0, 2, 4, 9])
    assert any(sorted(c for c in r[2:] if c >= 0) == [2, 9] for r in rows)
    assert all(set(c for c in r[2:] if c >= 0) <= {2, 9} for r in rows)


def test_a_removed_chunk_does_not_come_back():
    for row in _rows(500, 4, 1.0, 3.0, 4, [3, 1, 6, 2], [0, 1, 2, 3, 4, 5, 6, 7]):
        kept = row[:4]
        added = [c for c in row if c >= 0 and c not in (3, 1, 6, 2)]
        assert set(c for c in row if c >= 0) == set(c for c in kept if c in (3, 1, 6, 2)) | set(added)
        assert set(added) <= {0, 4, 5, 7}


@pytest.mark.parametrize("causal", [True, False])
def test_candidates_follow_the_routing_masks(causal):
    """The candidate list is the set routing itself may select from: with k >= the
    number of candidates, routing returns exactly that set."""
    lay = mi.random_layout(4, n_chunks=14, max_len=9, n_shots=3)
    L = mo.OracleLayout.from_layout(lay)
    rng = np.random.default_rng(0)
    q = rng.standard_normal((1, 1, L.N, 8))
    kbar = mo.pool(L, rng.standard_normal((1, 1, L.N, 8)))
    sel, _ = mo.route(L, q, kbar, 14, causal)
    for i in range(L.N):
        assert sorted(int(c) for c in sel[0, 0, i] if c >= 0) == mp.candidates_of(L, i, causal)


def test_layer_level_wrapper_uses_one_stream_per_head_and_query():
    lay = mi.random_layout(2, n_chunks=10, max_len=6, n_shots=2)
    L = mo.OracleLayout.from_layout(lay)
    rng = np.random.default_rng(5)
    q = rng.standard_normal((1, 3, L.N, 8))
    kbar = mo.pool(L, rng.standard_normal((1, 3, L.N, 8)))
    sel, _ = mo.route(L, q, kbar, 3, True)
    full = mp.perturb(L, sel, 3, True, 1.0, 1.0, 2, seed=99)
    assert full.shape == (1, 3, L.N, 5)
    qidx = np.array([L.N - 1, 3, L.N // 2])
    part = mp.perturb(L, sel[:, 1:2, qidx], 3, True, 1.0, 1.0, 2, seed=99, qidx=qidx, heads=[1], H=3)
    assert (part[0, 0] == full[0, 1, qidx]).all()
    assert (mp.perturb(L, sel, 3, True, 1.0, 1.0, 2, seed=100) != full).any()
