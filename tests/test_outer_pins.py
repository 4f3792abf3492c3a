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


def test_segments_cut_at_captions_and_shots():
    """Expected values written out by hand: 3 shots of [caption 8 | 2 frames x 16 tokens in chunks of 8]."""
    import moc_inputs as mi
    lay = mi.multishot_layout(3, 8, 2, 16, 8, "frame")
    seg, cap = ou.segments(lay.offsets, lay.shot, lay.text_spans)
    assert seg.tolist() == [0, 8, 40, 48, 80, 88, 120] and cap.tolist() == [1, 0, 1, 0, 1, 0]
    # no captions: one segment per shot; a caption of two chunks is still one segment
    seg, cap = ou.segments([0, 4, 8, 12, 20], [0, 0, 1, 1], np.zeros((0, 2), int))
    assert seg.tolist() == [0, 8, 20] and cap.tolist() == [0, 0]
    seg, cap = ou.segments([0, 4, 8, 12, 20], [0, 0, 0, 0], [[0, 8]])
    assert seg.tolist() == [0, 8, 20] and cap.tolist() == [1, 0]


def test_reduced_layout_by_hand_and_by_row_bookkeeping():
    import moc_inputs as mi
    lay = mi.multishot_layout(3, 8, 2, 16, 8, "frame")
    seg, _ = ou.segments(lay.offsets, lay.shot, lay.text_spans)
    kept = [0, 2, 4, 5]
    red = ou.reduce_layout(lay.offsets, lay.shot, lay.window, lay.text_spans, seg, kept)
    # by hand: three captions of 8 tokens, then the last shot's 4 video chunks of 8
    assert red["offsets"].tolist() == [0, 8, 16, 24, 32, 40, 48, 56]
    assert red["shot"].tolist() == [0, 1, 2, 2, 2, 2, 2]
    assert red["text_spans"].tolist() == [[0, 8], [8, 16], [16, 24]]
    assert red["window"].tolist() == [lay.window[j] for j in (0, 5, 10, 11, 12, 13, 14)]
    # every reduced chunk is an original chunk moved as a whole (checked through the row map)
    rows = ou.reduced_rows(seg, kept)
    assert int(red["offsets"][-1]) == len(rows)
    src_chunk = np.searchsorted(lay.offsets, rows[red["offsets"][:-1]], side="right") - 1
    assert (np.diff(red["offsets"]) == np.diff(lay.offsets)[src_chunk]).all()
    assert (red["shot"] == lay.shot[src_chunk]).all() and (red["window"] == lay.window[src_chunk]).all()
    # a caption span cut by a segment boundary keeps only the part inside the kept segment
    red = ou.reduce_layout([0, 4, 8, 12], [0, 0, 0], None, [[0, 8]], [0, 4, 12], [1])
    assert red["offsets"].tolist() == [0, 4, 8] and red["text_spans"].tolist() == [[0, 4]]
    assert red["window"].tolist() == [1, 2]
    with pytest.raises(ValueError):
        ou.reduce_layout(lay.offsets, lay.shot, lay.window, lay.text_spans, np.array([0, 12, 120]), [0])


def test_host_layout_calls_agree_with_the_oracle_bookkeeping():
    """moc_outer_segments / moc_reduce_layout (host-only entry points of the library) against the
    oracle's independent versions on irregular layouts."""
    import moc_inputs as mi
    from paper_2508_21058_amd import binding as mb
    for seed in range(12):
        lay = mi.random_layout(400 + seed, n_chunks=14, max_len=9, n_shots=1 + seed % 4, text_prob=0.3,
                               window=["mixed", "chunk", "shot"][seed % 3])
        seg_o, cap_o = ou.segments(lay.offsets, lay.shot, lay.text_spans)
        seg_l, cap_l = mb.outer_segments(lay.offsets, lay.shot, lay.text_spans)
        assert seg_l.tolist() == seg_o.tolist() and cap_l.tolist() == cap_o.tolist()
        rng = np.random.default_rng(seed)
        P = len(seg_o) - 1
        kept = sorted(rng.choice(P, size=int(rng.integers(1, P + 1)), replace=False).tolist())
        red = ou.reduce_layout(lay.offsets, lay.shot, lay.window, lay.text_spans, seg_o, kept)
        off, shot, win, spans, ranges = mb.reduce_layout(lay.offsets, lay.shot, lay.window, lay.text_spans, seg_l, kept)
        assert off.tolist() == red["offsets"].tolist() and shot.tolist() == red["shot"].tolist()
        assert win.tolist() == red["window"].tolist() and spans.tolist() == red["text_spans"].tolist()
        assert ranges.tolist() == [[int(seg_o[j]), int(seg_o[j + 1] - seg_o[j])] for j in kept]
    # errors: a segment boundary inside a chunk, kept out of order
    lay = mi.multishot_layout(2, 8, 2, 16, 8, "frame")
    with pytest.raises(mb.MocError):
        mb.reduce_layout(lay.offsets, lay.shot, lay.window, lay.text_spans, [0, 12, lay.N], [0])
    with pytest.raises(mb.MocError):
        mb.reduce_layout(lay.offsets, lay.shot, lay.window, lay.text_spans, [0, 8, 40, lay.N], [1, 0])
