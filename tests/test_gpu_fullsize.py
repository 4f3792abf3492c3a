"""Parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (all heads, bf16, same seeded device-generated inputs), on sampled
outputs the oracle can compute one by one:

  - pooled keys of one head, all chunks;
  - selections of one head, all N queries (tie tolerance as in the small tests);
  - o, lse, dq at sampled queries of that head;
  - dk, dv at all tokens of sampled chunks of that head; for the single-shot,
    both eight-shot and one sweep case also a caption chunk, whose keys are
    attended by all N queries (then o and lse are compared on the whole head).

The head checked has the oracle's selection injected before the attention
calls, so no tie can leak into the attention comparison.
"""
import numpy as np
import pytest
import torch

import moc_inputs as mi
from oracle import moc_oracle as mo
from paper_2508_21058_amd import binding as mb
from tests.test_gpu_parity import check_close, check_sel

pytestmark = pytest.mark.gpu


def _run(workload, window, head, n_sample, with_text_chunk, seed=1234, chunk=None, lay=None, cfg=None, n_chunks=2,
         topk=None, pick_chunks=None):
    cfg = dict(cfg or mi.CONFIGS[workload])
    if topk is not None:
        cfg["topk"] = topk
    lay = lay or mi.config_layout(workload, window=window, chunk=chunk)
    B, H, d, topk, N = cfg["B"], cfg["H"], cfg["d"], cfg["topk"], lay.N
    causal = bool(cfg.get("causal", True))
    q, k, v, d_o = (t.to(torch.bfloat16).contiguous() for t in mi.qkv_do(B, H, N, d, seed, "cuda"))
    meta = mb.chunk_meta(lay.offsets, lay.shot, lay.window, lay.text_spans)
    pooled, sel = mb.route(meta, q, k, topk, causal)
    torch.cuda.synchronize()

    L = mo.OracleLayout.from_layout(lay)
    f64 = lambda t: t[0:1, head:head + 1].float().cpu().numpy().astype(np.float64)
    qn, kn, vn, don = f64(q), f64(k), f64(v), f64(d_o)

    # stage b: pooled keys
    kbar = mo.pool(L, kn)
    err = np.abs(pooled[0, head].cpu().numpy() - kbar[0, 0]).max() / np.abs(kbar).max()
    assert err <= 1e-5, f"pooled keys rel err {err:.3e}"

    # stage c: selections of the whole head
    sel_ref, _ = mo.route(L, qn, kbar, topk, causal)
    sel_gpu = sel[0, head].cpu().numpy()
    # every row that differs anywhere (set or order) must be explained by ties in the oracle's scores
    bad = np.nonzero((sel_gpu != sel_ref[0, 0]).any(-1))[0].astype(np.int32)
    if len(bad):
        assert len(bad) <= max(2, N // 2000), f"{len(bad)} rows differ"
        _, sc, _ = mo.route(L, qn, kbar, topk, causal, bad, want_scores=True)
        check_sel(sel_gpu[bad], sel_ref[0, 0][bad], sc[0, 0], topk)

    # stage d with the oracle's selection for this head
    sel[0, head] = torch.from_numpy(sel_ref[0, 0]).to("cuda")
    ws = mb.attn_workspace(meta, B, H, d, topk, torch.bfloat16, True)
    o, lse = mb.attn_fwd(meta, q, k, v, sel, None, ws)
    dq, dk, dv = mb.attn_bwd(meta, q, k, v, o, lse, d_o, sel, None, ws, None, after_fwd=True)    # as bench.py's step
    torch.cuda.synchronize()

    rng = np.random.default_rng(5)
    video = np.nonzero(L.kind == 0)[0]
    chunks = list(pick_chunks) if pick_chunks is not None else \
        list(rng.choice(video[len(video) // 3:], size=n_chunks, replace=False))
    if with_text_chunk:
        chunks.append(int(np.nonzero(L.kind == 1)[0][0]))
    chunks = np.array(sorted(chunks), dtype=np.int32)
    att = np.zeros(N, bool)
    for j in chunks:
        if L.kind[j] == 0:
            att |= (L.win[L.chunk_of] == L.win[j]) | (sel_ref[0, 0] == j).any(-1)
    extra = rng.choice(N, size=n_sample, replace=False)
    # last queries, first queries, a caption query and random ones are always sampled
    att[extra] = True
    att[[0, 1, N - 1, N - 2]] = True
    qidx = np.nonzero(att)[0].astype(np.int32)

    sel_s = sel_ref[:, :, qidx]
    if with_text_chunk:
        # a caption chunk is attended by every query: its dK / dV need o and lse of the whole head, so the
        # forward is compared on all N queries; dQ stays on the sample
        o_all, lse_all, _ = mo.attn_fwd(L, qn, kn, vn, sel_ref)
        check_close("o", o[0, head].float().cpu().numpy(), o_all[0, 0])
        check_close("lse", lse[0, head].cpu().numpy(), lse_all[0, 0])
        o_ref, lse_ref = o_all[:, :, qidx], lse_all[:, :, qidx]
        o_full, lse_full = o_all, lse_all
    else:
        o_ref, lse_ref, _ = mo.attn_fwd(L, qn, kn, vn, sel_s, None, qidx)
        check_close("o", o[0, head].float().cpu().numpy()[qidx], o_ref[0, 0])
        check_close("lse", lse[0, head].cpu().numpy()[qidx], lse_ref[0, 0])
        o_full = np.zeros((1, 1, N, d)); o_full[0, 0, qidx] = o_ref[0, 0]
        lse_full = np.zeros((1, 1, N)); lse_full[0, 0, qidx] = lse_ref[0, 0]
    dq_ref = mo.attn_bwd_dq(L, qn, kn, vn, sel_s, o_ref, lse_ref, don[:, :, qidx], None, qidx)
    check_close("dq", dq[0, head].float().cpu().numpy()[qidx], dq_ref[0, 0])

    dk_ref, dv_ref = mo.attn_bwd_dkdv(L, qn, kn, vn, sel_ref, o_full, lse_full, don, None, chunks)
    rows = np.concatenate([np.arange(L.off[j], L.off[j + 1]) for j in chunks])
    check_close("dk", dk[0, head].float().cpu().numpy()[rows], dk_ref[0, 0][rows])
    check_close("dv", dv[0, head].float().cpu().numpy()[rows], dv_ref[0, 0][rows])
    meta.close()


def test_single_shot_config_forward_backward():
    """Single-shot configuration: 512 text + 21 x 1560 tokens, chunk 260, frame window, k=5, H=24, d=128."""
    _run("single", None, head=5, n_sample=384, with_text_chunk=True)


def test_eight_shot_config_frame_window():
    """Eight-shot configuration (benchmark workload): 8 x (256 + 9 x 1560) tokens, frame window, k=8."""
    _run("eight", "frame", head=17, n_sample=384, with_text_chunk=True)


def test_eight_shot_config_shot_window():
    """Config 4 with the whole shot as the forced local window (the multi-shot reading)."""
    _run("eight", "shot", head=2, n_sample=256, with_text_chunk=True)


def test_sweep_config_chunk_130():
    """Sweep configuration (32 shots, N = 457,472) at chunk 130: 3,488 chunks, 2-key tail tiles, k=8."""
    _run("sweep", "frame", head=7, n_sample=192, with_text_chunk=False, chunk=130)


def test_sweep_config_chunk_520():
    """Config 5 at chunk 520: chunks longer than the chunk-resident routed forward takes (tiled routed path), 8-key tails."""
    _run("sweep", "frame", head=11, n_sample=192, with_text_chunk=False, chunk=520)


def test_single_shot_training_setup_non_causal():
    """App. "Training Details", single-shot model: ~6.3k tokens, chunk 256 (ragged last chunk of 112),
    own-chunk window, k=3, no causal mask: candidates on both sides of the query."""
    _run("short", None, head=9, n_sample=512, with_text_chunk=True, n_chunks=3)


def test_multi_shot_training_setup_chunk_1280():
    """App. "Training Details", multi-shot model at its final chunk size: 8 x (256 text + 14,040 video),
    chunks of 1280 with a ragged 1240 tail per shot, whole-shot window, k=5."""
    _run("paper", None, head=3, n_sample=128, with_text_chunk=False, chunk=1280)


def test_multi_shot_training_setup_chunk_2560():
    _run("paper", None, head=20, n_sample=128, with_text_chunk=False, chunk=2560, n_chunks=1)


def test_chunks_of_10240_tokens():
    """The largest chunk size of the multi-shot schedule on a two-shot stream: fewer candidates (2)
    than k (5), every routed list covers a whole shot, 80 key tiles share one chunk's query list."""
    lay = mi.stream_layout(2, 64, 12000, 10240, "shot")
    cfg = dict(B=1, H=2, d=128, dtype="bf16", topk=5)
    _run(None, None, head=1, n_sample=64, with_text_chunk=False, lay=lay, cfg=cfg, n_chunks=1)


def test_sweep_config_chunk_260_k16():
    """Sweep configuration at its widest selection: 16 routed chunks per query, rows of 16 slots."""
    _run("sweep", "frame", head=19, n_sample=128, with_text_chunk=False, chunk=260, topk=16, n_chunks=1)


def test_sweep_config_chunk_260_k2():
    """... and at its narrowest, with a caption chunk among the sampled key chunks: its 256 keys are attended by
    all 457,472 queries (56 query segments of partial sums and the fixed-order reduction)."""
    _run("sweep", "frame", head=4, n_sample=128, with_text_chunk=True, chunk=260, topk=2, n_chunks=1)


def test_eight_shot_stream_of_180k_tokens_with_mixed_chunk_sizes():
    """The paper's 8-shot scale (Sec. 3.3 worked example: ~180k tokens, k=5): 8 x (256 text + 22,464 video)
    = 181,760 tokens, chunks of 10240 / 5120 / 2560 / 1280 tokens side by side in one stream (ragged tails),
    whole-shot window. Chunks of every size are among the sampled key chunks."""
    lay = mi.config_layout("long")
    lens = np.diff(lay.offsets)
    assert lay.N == 181760 and {10240, 5120, 2560, 1280} <= set(lens.tolist())
    video = [j for j in range(lay.C // 2, lay.C) if lens[j] != 256]
    pick = [next(j for j in video if lens[j] == m) for m in (10240, 5120, 2560, 1280)]
    _run("long", None, head=13, n_sample=96, with_text_chunk=False, pick_chunks=pick)
