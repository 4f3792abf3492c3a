"""Pins of the outer-loop routing oracle (App. "Outer Loop Context Routing")."""
import itertools

import numpy as np
import pytest

from oracle import moc_outer as ou


def _stream(seed, P=7, D=12, max_len=9):
    rng = np.random.default_rng(seed)
    lens = rng.integers(1, max_len + 1, size=P)
    off = np.concatenate([[0], np.cumsum(lens)])
    return rng.standard_normal((off[-1], D)), off


def test_means_by_explicit_loops():
    x, off = _stream(0)
    m = ou.segment_means(x, off)
    for j in range(len(off) - 1):
        for c in range(x.shape[1]):
            s = 0.0
            for r in range(off[j], off[j + 1]):
                s += x[r, c]
            assert abs(m[j, c] - s / (off[j + 1] - off[j])) < 1e-12


def test_constant_segments_give_closed_form_scores():
    # every token of segment j equals a_j * e_1 + e_2: the score against g is a_j a_g + 1
    a = np.array([0.5, -2.0, 3.0, 1.0, 0.25])
    off = np.array([0, 3, 4, 9, 11, 15])
    x = np.zeros((15, 4))
    for j in range(5):
        x[off[j]:off[j + 1], 0] = a[j]
        x[off[j]:off[j + 1], 1] = 1.0
    sel, scores, kept, _ = ou.outer_route(x, off, None, g=4, M=2, causal=True)
    assert np.allclose(scores, a * a[4] + 1)
    assert sel.tolist() == [2, 3] and kept == [2, 3, 4]
    sel, _, kept, _ = ou.outer_route(x, off, [1, 0, 0, 0, 0], g=2, M=3, causal=False)
    # a_j * 3 + 1: segment 3 (4.0), segment 4 (1.75), segment 1 (-5); segment 0 is mandatory, not a candidate
    assert sel.tolist() == [3, 4, 1] and kept == [0, 1, 2, 3, 4]


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("causal", [True, False])
def test_top_m_is_the_subset_with_the_largest_score_sum(seed, causal):
    """The appendix defines the selection as the size-M subset maximising the summed score."""
    x, off = _stream(seed)
    P = len(off) - 1
    rng = np.random.default_rng(seed + 100)
    mand = (rng.random(P) < 0.25).astype(np.int32)
    g = int(rng.integers(1, P))
    mand[g] = 0
    for M in (1, 2, 3):
        sel, scores, kept, _ = ou.outer_route(x, off, mand, g, M, causal)
        cand = [j for j in range(P) if j != g and not mand[j] and (not causal or j < g)]
        m_eff = min(M, len(cand))
        got = [int(j) for j in sel if j >= 0]
        assert len(got) == m_eff and (sel[m_eff:] == -1).all()
        best = max(itertools.combinations(cand, m_eff), key=lambda c: sum(scores[j] for j in c)) if m_eff else ()
        assert abs(sum(scores[j] for j in got) - sum(scores[j] for j in best)) < 1e-12
        assert all(scores[got[t]] >= scores[got[t + 1]] for t in range(len(got) - 1))      # best first
        assert kept == sorted(set(got) | set(np.nonzero(mand)[0]) | {g})


def test_ties_go_to_the_lower_index_and_short_history_takes_all():
    off = np.array([0, 2, 4, 6, 8])
    x = np.ones((8, 3))
    sel, _, kept, _ = ou.outer_route(x, off, None, g=3, M=2, causal=True)
    assert sel.tolist() == [0, 1] and kept == [0, 1, 3]
    sel, _, kept, _ = ou.outer_route(x, off, None, g=1, M=3, causal=True)
    assert sel.tolist() == [0, -1, -1] and kept == [0, 1]
    sel, _, kept, _ = ou.outer_route(x, off, None, g=0, M=2, causal=True)
    assert sel.tolist() == [-1, -1] and kept == [0]


def test_reduced_rows_keep_stream_order():
    off = np.array([0, 3, 4, 9, 11])
    rows = ou.reduced_rows(off, [0, 2, 3])
    assert rows.tolist() == [0, 1, 2, 4, 5, 6, 7, 8, 9, 10]
    assert (np.diff(rows) > 0).all()


def test_segments_and_reduced_layout_bookkeeping():
    """Layout helpers used with the outer loop: captions are segments of their own, a shot's video chunks
    form one segment, and the reduced layout keeps chunk lengths, shots, windows and caption spans."""
    import moc_inputs as mi
    lay = mi.multishot_layout(3, 8, 2, 16, 8, "frame")
    seg, cap = mi.shot_segments(lay)
    assert seg.tolist() == [0, 8, 40, 48, 80, 88, 120] and cap.tolist() == [1, 0, 1, 0, 1, 0]
    kept = [0, 2, 4, 5]
    red = mi.reduce_layout(lay, seg, kept)
    rows = ou.reduced_rows(seg, kept)
    assert red.N == len(rows) == 8 + 8 + 8 + 32
    # every reduced chunk is an original chunk, moved as a whole
    src_chunk = np.searchsorted(lay.offsets, rows[red.offsets[:-1]], side="right") - 1
    assert (np.diff(red.offsets) == np.diff(lay.offsets)[src_chunk]).all()
    assert (red.shot == lay.shot[src_chunk]).all() and (red.window == lay.window[src_chunk]).all()
    assert red.text_spans.tolist() == [[0, 8], [8, 16], [16, 24]]
    with pytest.raises(ValueError):
        mi.reduce_layout(lay, np.array([0, 12, 120], np.int32), [0])     # 12 is not a chunk boundary
