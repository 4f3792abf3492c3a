"""Parity of the outer-loop routing (App. "Outer Loop Context Routing") and of the row gather that builds
the reduced stream. Means and scores are fp32 sums of exact inputs: tolerance 1e-5 of the largest
magnitude; selections identical except for ties within 1e-5 of the largest score; the gather is exact."""
import numpy as np
import pytest
import torch

import moc_inputs as mi
from oracle import moc_oracle as mo
from oracle import moc_outer as ou
from paper_2508_21058_amd import binding as mb
from tests.test_gpu_parity import check_close, to_dev

pytestmark = pytest.mark.gpu


def _check_route(x_t, off, mand, g, M, causal):
    xn = x_t.float().cpu().numpy().astype(np.float64)
    sel_ref, sc_ref, kept_ref, means_ref = ou.outer_route(xn, off, mand, g, M, causal)
    mean, scores, sel, kept = mb.outer_route(x_t, off, mand, g, M, causal)
    torch.cuda.synchronize()
    m = mean.cpu().numpy().astype(np.float64)
    assert np.abs(m - means_ref).max() <= 1e-5 * max(np.abs(means_ref).max(), 1e-30)
    s = scores.cpu().numpy().astype(np.float64)
    tol = 1e-5 * max(np.abs(sc_ref).max(), 1e-30)
    assert np.abs(s - sc_ref).max() <= tol
    if not np.array_equal(sel, sel_ref):                       # only ties may differ
        a, b = set(sel[sel >= 0].tolist()), set(sel_ref[sel_ref >= 0].tolist())
        assert len(a) == len(b)
        kth = min(sc_ref[j] for j in b)
        assert all(abs(sc_ref[j] - kth) <= tol for j in a ^ b)
    else:
        assert kept == kept_ref
    P = len(off) - 1
    mset = set(np.nonzero(mand)[0].tolist()) if mand is not None else set()
    assert kept == sorted(set(sel[sel >= 0].tolist()) | mset | {g})
    return sel, kept


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("D", [8, 264, 2056])
def test_ragged_segments(dtype, D):
    lens = [1, 63, 64, 65, 200, 7, 129, 640, 3]
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    x = mi.randn((int(off[-1]), D), 3, "cpu", bf16_round=True)
    x_t = to_dev(x.numpy(), dtype)
    mand = np.array([0, 0, 1, 0, 0, 0, 0, 0, 0], np.int32)
    for g, M, causal in [(8, 3, True), (4, 2, True), (4, 5, False), (0, 2, True), (1, 4, True), (7, 0, True)]:
        _check_route(x_t, off, mand if g != 2 else None, g, M, causal)
    _check_route(x_t, off, None, 5, 9, False)


def test_equal_segments_tie_to_the_lower_index():
    off = np.arange(0, 9 * 70, 70).astype(np.int32)
    x_t = torch.ones(int(off[-1]), 16, dtype=torch.bfloat16, device="cuda")
    sel, kept = _check_route(x_t, off, None, 7, 3, True)
    assert sel.tolist() == [0, 1, 2] and kept == [0, 1, 2, 7]


def test_gather_is_exact_on_head_major_and_flat_tensors():
    rng = np.random.default_rng(0)
    src = torch.randn(2, 3, 500, 64, device="cuda").to(torch.bfloat16)
    ranges = [(490, 10), (0, 1), (17, 130), (300, 64)]
    rows = np.concatenate([np.arange(s, s + n) for s, n in ranges])
    got = mb.gather_rows(src, ranges)
    assert torch.equal(got, src[:, :, torch.from_numpy(rows).cuda()])
    flat = torch.randn(777, 40, device="cuda")
    got = mb.gather_rows(flat, [(5, 700), (0, 5)])
    assert torch.equal(got, torch.cat([flat[5:705], flat[0:5]]))
    # empty ranges add nothing, overlapping ranges repeat their rows
    got = mb.gather_rows(flat, [(9, 0), (5, 3), (777, 0), (6, 3), (0, 0)])
    assert torch.equal(got, torch.cat([flat[5:8], flat[6:9]]))
    assert mb.gather_rows(flat, [(9, 0)]).shape == (0, 40)


def test_full_size_stream_of_the_benchmark_layout():
    """N = 114,368 tokens, D = H d = 3072 (bf16, 703 MB): captions mandatory, shots compete."""
    lay = mi.config_layout("eight")
    seg, cap = mb.outer_segments(lay.offsets, lay.shot, lay.text_spans)
    seg_o, cap_o = ou.segments(lay.offsets, lay.shot, lay.text_spans)
    assert seg.tolist() == seg_o.tolist() and cap.tolist() == cap_o.tolist()
    D = 3072
    x = mi.randn((lay.N, D), 99, "cuda").to(torch.bfloat16).contiguous()
    sel, kept = _check_route(x, seg, cap, 15, 3, True)
    assert len(kept) == 8 + 3 + 1
    ranges = [(int(seg[j]), int(seg[j + 1] - seg[j])) for j in kept]
    red = mb.gather_rows(x, ranges)
    rows = torch.from_numpy(ou.reduced_rows(seg, kept)).cuda()
    assert torch.equal(red, x[rows])


def test_reduced_stream_feeds_the_inner_layer():
    """Outer selection -> reduced q, k, v, dO and layout -> inner layer; everything is compared with the
    oracle run on the oracle's own reduced stream."""
    lay = mi.multishot_layout(4, 16, 3, 64, 32, "frame")
    H, d, topk, M = 2, 64, 2, 1
    N = lay.N
    q, k, v, d_o = mi.qkv_do(1, H, N, d, 17, "cpu", bf16_round=True)
    # features of the outer router: the per-head keys side by side, [N, H d]
    feat = k[0].permute(1, 0, 2).reshape(N, H * d).contiguous()

    # oracle side: its own segments, selection, reduced rows and reduced layout
    seg_o, cap_o = ou.segments(lay.offsets, lay.shot, lay.text_spans)
    g = len(seg_o) - 2
    sel_ref, _, kept_ref, _ = ou.outer_route(feat.numpy().astype(np.float64), seg_o, cap_o, g, M, True)
    rows = ou.reduced_rows(seg_o, kept_ref)
    red_o = ou.reduce_layout(lay.offsets, lay.shot, lay.window, lay.text_spans, seg_o, kept_ref)
    L = mo.OracleLayout(red_o["offsets"], red_o["window"], red_o["text_spans"])
    qn, kn, vn, don = (t.numpy().astype(np.float64)[:, :, rows] for t in (q, k, v, d_o))
    ref = mo.moc_layer(L, qn, kn, vn, topk, True, don)

    # library side: its own segments, selection, gather table and reduced layout
    seg, cap = mb.outer_segments(lay.offsets, lay.shot, lay.text_spans)
    _, _, sel, kept = mb.outer_route(to_dev(feat.numpy(), torch.bfloat16), seg, cap, g, M, True)
    assert kept == kept_ref and sel.tolist() == sel_ref.tolist()
    r_off, r_shot, r_win, r_spans, ranges = mb.reduce_layout(lay.offsets, lay.shot, lay.window, lay.text_spans, seg, kept)
    qd, kd, vd, dod = (mb.gather_rows(to_dev(t.numpy(), torch.bfloat16), ranges) for t in (q, k, v, d_o))
    meta = mb.chunk_meta(r_off, r_shot, r_win, r_spans)
    _, isel = mb.route(meta, qd, kd, topk, True)
    assert (np.sort(isel.cpu().numpy(), -1) == np.sort(ref["sel"], -1)).all()
    o, lse = mb.attn_fwd(meta, qd, kd, vd, isel)
    dq, dk, dv = mb.attn_bwd(meta, qd, kd, vd, o, lse, dod, isel)
    torch.cuda.synchronize()
    for name, got in (("o", o), ("dq", dq), ("dk", dk), ("dv", dv)):
        check_close(name, got.float().cpu().numpy(), ref[name])
    meta.close()
