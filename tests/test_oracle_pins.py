"""Pins for the CPU oracle: nothing here compares the oracle with itself.

1. brute force with an explicit N x N mask + torch autograd (tests/bruteforce.py)
2. reductions to textbook attention (torch SDPA on CPU)
3. structural invariants of the routing rule
4. central finite differences for the backward
5. closed-form pair counts / the FLOP figure the paper prints
"""
import json
import os

import numpy as np
import pytest
import torch

import moc_inputs as mi
from oracle import moc_oracle as mo
from tests import bruteforce as bf

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _run_oracle(lay, q, k, v, topk, causal=True, d_o=None):
    L = mo.OracleLayout.from_layout(lay)
    r = mo.moc_layer(L, q[None, None], k[None, None], v[None, None], topk, causal,
                     None if d_o is None else d_o[None, None])
    return {key: (val[0, 0] if isinstance(val, np.ndarray) else val) for key, val in r.items()}


def _assert_sel_equal(sel_o, sel_b):
    assert sel_o.shape == sel_b.shape
    assert np.array_equal(sel_o.astype(np.int64), sel_b.astype(np.int64))


# ---------------------------------------------------------------- 1. brute force

LAYOUTS = [("tiny", None)] + [(f"rand{s}", s) for s in range(8)]


@pytest.mark.parametrize("name,seed", LAYOUTS)
@pytest.mark.parametrize("causal", [True, False])
def test_bruteforce_forward_backward(name, seed, causal):
    if seed is None:
        lay, d, topk = mi.config_layout("tiny"), 64, 2
    else:
        win = ["mixed", "chunk", "shot"][seed % 3]
        lay = mi.random_layout(seed, n_chunks=10 + seed, max_len=24, n_shots=1 + seed % 3, window=win)
        d, topk = 16, 1 + seed % 4
    N = lay.N
    q, k, v, d_o = (_rand((N, d), 100 + 10 * (seed or 0) + i) for i in range(4))
    ref = bf.moc_bruteforce(lay, q, k, v, topk, causal, d_o)
    got = _run_oracle(lay, q, k, v, topk, causal, d_o)
    np.testing.assert_allclose(got["kbar"], ref["kbar"], rtol=1e-12, atol=1e-13)
    _assert_sel_equal(got["sel"], ref["sel"])
    for key in ("o", "lse", "dq", "dk", "dv"):
        np.testing.assert_allclose(got[key], ref[key], rtol=1e-6, atol=1e-9, err_msg=key)
    assert got["n_pairs"] == int(ref["mask"].sum())
    assert got["n_eligible"] == int(np.isfinite(ref["scores"]).sum())


def test_chunk_tables_match_bucketize():
    for seed in range(5):
        lay = mi.random_layout(seed, n_chunks=15, max_len=9, n_shots=3)
        L = mo.OracleLayout.from_layout(lay)
        off, C, N, chunk_of, is_text, win = bf.chunk_tables(lay)
        assert np.array_equal(L.chunk_of, chunk_of)
        assert np.array_equal(L.kind.astype(bool), is_text)


def test_ties_pick_lowest_index():
    """Identical chunks give identical scores: the lower chunk index must win."""
    lay = mi.multishot_layout(1, 0, 6, 4, 4, "chunk")       # 6 chunks of 4 tokens, no text
    d = 8
    base = _rand((4, d), 7)
    k = np.concatenate([base] * 6)                           # every chunk has the same keys
    q, v = _rand((lay.N, d), 8), _rand((lay.N, d), 9)
    got = _run_oracle(lay, q, k, v, 2)
    for i in range(lay.N):
        c = i // 4
        want = [j for j in range(c)][:2] + [-1] * (2 - min(2, c))
        assert list(got["sel"][i]) == want


# ---------------------------------------------------------------- 2. reductions

def _sdpa(q, k, v, **kw):
    t = lambda a: torch.tensor(a, dtype=torch.float64)[None, None]
    return torch.nn.functional.scaled_dot_product_attention(t(q), t(k), t(v), **kw)[0, 0].numpy()


def test_single_window_is_dense_attention():
    lay = mi.multishot_layout(1, 8, 3, 12, 4, "shot")        # caption + all frames in one window
    d = 16
    q, k, v = (_rand((lay.N, d), 20 + i) for i in range(3))
    got = _run_oracle(lay, q, k, v, 3)
    np.testing.assert_allclose(got["o"], _sdpa(q, k, v), rtol=1e-9, atol=1e-12)
    assert (got["sel"] == -1).all()                          # nothing left to route to


def test_token_chunks_full_k_is_causal_attention():
    N, d = 48, 8
    lay = mi.multishot_layout(1, 0, 1, N, 1, "chunk")        # chunk length 1, no text
    q, k, v = (_rand((N, d), 30 + i) for i in range(3))
    got = _run_oracle(lay, q, k, v, N)
    np.testing.assert_allclose(got["o"], _sdpa(q, k, v, is_causal=True), rtol=1e-9, atol=1e-12)


def test_full_k_is_block_causal():
    lay = mi.config_layout("tiny")
    d = 16
    N, C = lay.N, lay.C
    q, k, v = (_rand((N, d), 40 + i) for i in range(3))
    got = _run_oracle(lay, q, k, v, C)
    chunk_of = np.repeat(np.arange(C), np.diff(lay.offsets))
    mask = torch.tensor(chunk_of[None, :] <= chunk_of[:, None])
    np.testing.assert_allclose(got["o"], _sdpa(q, k, v, attn_mask=mask), rtol=1e-9, atol=1e-12)


def test_k0_is_block_diagonal_plus_text():
    lay = mi.multishot_layout(2, 6, 2, 10, 5, "frame")
    d = 8
    N, C = lay.N, lay.C
    q, k, v = (_rand((N, d), 50 + i) for i in range(3))
    got = _run_oracle(lay, q, k, v, 0)
    off, C, N, chunk_of, is_text, win = bf.chunk_tables(lay)
    mask = is_text[chunk_of][None, :] | (win[chunk_of][None, :] == win[chunk_of][:, None])
    np.testing.assert_allclose(got["o"], _sdpa(q, k, v, attn_mask=torch.tensor(mask)), rtol=1e-9, atol=1e-12)


# ---------------------------------------------------------------- 3. invariants

@pytest.mark.parametrize("seed", range(4))
def test_routing_invariants(seed):
    lay = mi.random_layout(100 + seed, n_chunks=20, max_len=12, n_shots=3)
    d, topk = 12, 3
    N, C = lay.N, lay.C
    q, k, v = (_rand((N, d), 60 + 3 * seed + i) for i in range(3))
    L = mo.OracleLayout.from_layout(lay)
    kbar = mo.pool(L, k[None, None])
    sel, n_el = mo.route(L, q[None, None], kbar, topk)
    sel = sel[0, 0]
    mand = bf.mandatory_matrix(lay)
    chunk_of = L.chunk_of
    for i in range(N):
        r = [j for j in sel[i] if j >= 0]
        n_elig = sum(1 for j in range(chunk_of[i]) if not mand[i, j])
        assert len(r) == min(topk, n_elig)                  # |R| = min(k, |E|)
        assert len(set(r)) == len(r)
        assert all(j < chunk_of[i] for j in r)              # never a later (or the own) chunk
        assert not any(mand[i, j] for j in r)               # k is not spent on forced links
        assert list(sel[i]) == r + [-1] * (topk - len(r))   # -1 padded at the end
    # nestedness: top-k is a prefix of top-(k+1)
    sel2, _ = mo.route(L, q[None, None], kbar, topk + 1)
    assert np.array_equal(sel2[0, 0][:, :topk], sel)
    # positive scaling of q leaves the selection unchanged
    sel3, _ = mo.route(L, 3.7 * q[None, None], kbar, topk)
    assert np.array_equal(sel3[0, 0], sel)
    # permuting tokens inside key chunks leaves sel and o unchanged
    rng = np.random.default_rng(seed)
    perm = np.concatenate([lay.offsets[j] + rng.permutation(lay.offsets[j + 1] - lay.offsets[j])
                           for j in range(C)])
    o1, lse1, _ = mo.attn_fwd(L, q[None, None], k[None, None], v[None, None], sel[None, None])
    kb2 = mo.pool(L, k[perm][None, None])
    sel4, _ = mo.route(L, q[None, None], kb2, topk)
    o2, lse2, _ = mo.attn_fwd(L, q[None, None], k[perm][None, None], v[perm][None, None], sel4)
    assert np.array_equal(sel4[0, 0], sel)
    np.testing.assert_allclose(o2, o1, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(lse2, lse1, rtol=1e-10, atol=1e-12)


def test_heads_are_independent():
    lay = mi.random_layout(5, n_chunks=12, max_len=10)
    d, topk, N = 8, 2, lay.N
    q, k, v = (_rand((1, 3, N, d), 70 + i) for i in range(3))
    L = mo.OracleLayout.from_layout(lay)
    full = mo.moc_layer(L, q, k, v, topk)
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[:, 0], k2[:, 0], v2[:, 2] = 5.0, -2.0, 9.0            # disturb heads 0 and 2
    other = mo.moc_layer(L, q2, k2, v2, topk)
    assert np.array_equal(full["sel"][0, 1], other["sel"][0, 1])
    assert np.array_equal(full["o"][0, 1], other["o"][0, 1])


def test_ds_rows_sum_to_zero_via_dq_of_constant_keys():
    """With all keys equal, every dS row sums to zero, so dq must vanish."""
    lay = mi.random_layout(9, n_chunks=9, max_len=7)
    d, N = 8, lay.N
    q, v, d_o = (_rand((N, d), 80 + i) for i in range(3))
    k = np.tile(_rand((1, d), 83), (N, 1))
    got = _run_oracle(lay, q, k, v, 2, True, d_o)
    assert np.abs(got["dq"]).max() < 1e-12


# ---------------------------------------------------------------- 3b. subset modes

@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("causal", [True, False])
def test_query_and_chunk_subsets_equal_the_rows_of_the_full_run(seed, causal):
    """The full-size GPU comparisons and the benchmark's CPU leg call the oracle on a list of queries
    (`qidx`) or of key chunks (`chunks`). Those modes must give exactly the rows of the whole-sequence
    run, which the brute-force tests above pin. For dK / dV the o and lse arrays are filled only at
    the queries that attend a listed chunk, as the callers do."""
    lay = mi.random_layout(500 + seed, n_chunks=14, max_len=11, n_shots=2, text_prob=0.25,
                           window=["mixed", "chunk", "shot", "mixed"][seed])
    d, topk, N = 8, 1 + seed, lay.N
    q, k, v, d_o = (_rand((1, 2, N, d), 130 + 4 * seed + i) for i in range(4))
    L = mo.OracleLayout.from_layout(lay)
    full = mo.moc_layer(L, q, k, v, topk, causal, d_o)
    rng = np.random.default_rng(seed)
    qidx = np.sort(rng.choice(N, size=max(3, N // 4), replace=False)).astype(np.int32)
    qidx[0], qidx[-1] = 0, N - 1                                       # first and last token always in
    qidx = np.unique(qidx)
    sel_s, scores, n_el = mo.route(L, q, full["kbar"], topk, causal, qidx, want_scores=True)
    assert np.array_equal(sel_s, full["sel"][:, :, qidx])
    _, scores_full, _ = mo.route(L, q, full["kbar"], topk, causal, want_scores=True)
    assert np.array_equal(np.nan_to_num(scores, nan=-7e77), np.nan_to_num(scores_full[:, :, qidx], nan=-7e77))
    o_s, lse_s, n_pairs = mo.attn_fwd(L, q, k, v, sel_s, None, qidx)
    assert np.array_equal(o_s, full["o"][:, :, qidx]) and np.array_equal(lse_s, full["lse"][:, :, qidx])
    dq_s = mo.attn_bwd_dq(L, q, k, v, sel_s, o_s, lse_s, d_o[:, :, qidx], None, qidx)
    assert np.array_equal(dq_s, full["dq"][:, :, qidx])
    # pair count of the subset = the explicit mask's count on those rows (head 0)
    ref = bf.moc_bruteforce(lay, q[0, 0], k[0, 0], v[0, 0], topk, causal)
    _, _, n0 = mo.attn_fwd(L, q[:, :1], k[:, :1], v[:, :1], sel_s[:, :1], None, qidx)
    assert n0 == int(ref["mask"][qidx].sum())

    chunks = np.sort(rng.choice(lay.C, size=3, replace=False)).astype(np.int32)
    if L.kind.any():
        chunks = np.unique(np.append(chunks, np.nonzero(L.kind)[0][0])).astype(np.int32)    # a caption chunk too
    rows = np.concatenate([np.arange(L.off[j], L.off[j + 1]) for j in chunks])
    o_part, lse_part = np.zeros_like(full["o"]), np.zeros_like(full["lse"])
    for h in range(2):
        att = np.zeros(N, bool)
        for j in chunks:
            att |= (L.kind[j] == 1) | (L.win[L.chunk_of] == L.win[j]) | (full["sel"][0, h] == j).any(-1)
        o_part[0, h, att], lse_part[0, h, att] = full["o"][0, h, att], full["lse"][0, h, att]
    dk_s, dv_s = mo.attn_bwd_dkdv(L, q, k, v, full["sel"], o_part, lse_part, d_o, None, chunks)
    assert np.array_equal(dk_s[:, :, rows], full["dk"][:, :, rows])
    assert np.array_equal(dv_s[:, :, rows], full["dv"][:, :, rows])
    other = np.setdiff1d(np.arange(N), rows)
    assert not dk_s[:, :, other].any() and not dv_s[:, :, other].any()


def test_selection_rows_are_read_as_sets():
    """A selection row handed to the attention functions may repeat a chunk or name a forced link;
    the attended set is the union, so the result equals that of the cleaned row (and the brute-force mask)."""
    lay = mi.multishot_layout(2, 6, 2, 10, 5, "frame")
    d, N = 8, lay.N
    q, k, v, d_o = (_rand((1, 1, N, d), 150 + i) for i in range(4))
    L = mo.OracleLayout.from_layout(lay)
    clean = np.full((1, 1, N, 3), -1, np.int32)
    dirty = np.full((1, 1, N, 3), -1, np.int32)
    text0 = int(np.nonzero(L.kind)[0][0])
    for i in range(N):
        own = L.chunk_of[i]
        far = [j for j in range(lay.C) if L.kind[j] == 0 and L.win[j] != L.win[own]]
        clean[0, 0, i, 0] = far[i % len(far)]
        dirty[0, 0, i] = [far[i % len(far)], text0 if i % 2 else own, far[i % len(far)]]
    a = mo.attn_fwd(L, q, k, v, clean)
    b = mo.attn_fwd(L, q, k, v, dirty)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and a[2] == b[2]
    mask = bf.token_mask(lay, clean[0, 0].astype(np.int64))
    ref = bf.dense_masked_attention(q[0, 0], k[0, 0], v[0, 0], mask, d_o[0, 0])
    np.testing.assert_allclose(b[0][0, 0], ref["o"], rtol=1e-9, atol=1e-12)
    dq = mo.attn_bwd_dq(L, q, k, v, dirty, b[0], b[1], d_o)
    dk, dv = mo.attn_bwd_dkdv(L, q, k, v, dirty, b[0], b[1], d_o)
    np.testing.assert_allclose(dq[0, 0], ref["dq"], rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(dk[0, 0], ref["dk"], rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(dv[0, 0], ref["dv"], rtol=1e-6, atol=1e-9)


# ---------------------------------------------------------------- 4. finite differences

@pytest.mark.parametrize("seed", range(3))
def test_backward_central_finite_differences(seed):
    lay = mi.random_layout(200 + seed, n_chunks=9, max_len=8, n_shots=2)
    d, topk, N = 8, 2, lay.N
    q, k, v, d_o = (_rand((1, 1, N, d), 90 + 4 * seed + i) for i in range(4))
    L = mo.OracleLayout.from_layout(lay)
    r = mo.moc_layer(L, q, k, v, topk, True, d_o)
    sel = r["sel"]
    eps = 1e-5
    rng = np.random.default_rng(seed)

    def f(qq, kk, vv):                                      # forward with the selection frozen
        o, _, _ = mo.attn_fwd(L, qq, kk, vv, sel)
        return float((o * d_o).sum())

    for name, grad in (("q", r["dq"]), ("k", r["dk"]), ("v", r["dv"])):
        u = rng.standard_normal(q.shape)
        args_p = dict(q=q, k=k, v=v)
        args_m = dict(q=q, k=k, v=v)
        args_p[name] = args_p[name] + eps * u
        args_m[name] = args_m[name] - eps * u
        fd = (f(args_p["q"], args_p["k"], args_p["v"]) - f(args_m["q"], args_m["k"], args_m["v"])) / (2 * eps)
        an = float((grad * u).sum())
        assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, fd, an)


def test_unfrozen_forward_has_same_derivative_away_from_ties():
    """Hard top-k is piecewise constant: re-routing after a tiny perturbation
    gives the same selection, hence the same directional derivative."""
    lay = mi.random_layout(300, n_chunks=8, max_len=6)
    d, topk, N = 8, 2, lay.N
    q, k, v, d_o = (_rand((1, 1, N, d), 110 + i) for i in range(4))
    L = mo.OracleLayout.from_layout(lay)
    r = mo.moc_layer(L, q, k, v, topk, True, d_o)
    eps = 1e-7
    u = np.random.default_rng(1).standard_normal(k.shape)
    rp = mo.moc_layer(L, q, k + eps * u, v, topk)
    rm = mo.moc_layer(L, q, k - eps * u, v, topk)
    assert np.array_equal(rp["sel"], r["sel"]) and np.array_equal(rm["sel"], r["sel"])
    fd = float(((rp["o"] - rm["o"]) * d_o).sum()) / (2 * eps)
    an = float((r["dk"] * u).sum())
    assert abs(fd - an) <= 1e-4 * max(1.0, abs(an))


# ---------------------------------------------------------------- 5. counts

def test_paper_dense_flops_example():
    with open(os.path.join(GOLDEN, "paper_flops.json")) as f:
        g = json.load(f)
    L_, d = g["L"], g["d"]
    assert abs(4 * L_ * L_ * d / g["dense_flops_printed"] - 1) < 0.01


@pytest.mark.parametrize("window", ["frame", "shot"])
def test_pair_counts_closed_form_eight_shot(window):
    """Sum |Omega(i)| on sampled queries of the 8-shot layout against the count
    that follows from the rule: all caption tokens + own window + min(k, #earlier
    non-mandatory chunks) * chunk length."""
    lay = mi.config_layout("eight", window=window)
    L = mo.OracleLayout.from_layout(lay)
    d, topk = 4, 8
    N = lay.N
    rng = np.random.default_rng(3)
    qidx = np.sort(rng.choice(N, size=96, replace=False)).astype(np.int32)
    q = _rand((1, 1, N, d), 5)
    k = _rand((1, 1, N, d), 6)
    kbar = mo.pool(L, k)
    sel, _ = mo.route(L, q, kbar, topk, True, qidx)
    _, _, n_pairs = mo.attn_fwd(L, q, k, k, sel, None, qidx)
    text, fr, ft, ch = 256, 9, 1560, 260
    per_shot = text + fr * ft
    want = 0
    for i in qidx:
        s, r = divmod(int(i), per_shot)
        if window == "frame":
            if r < text:                       # caption query: all captions (own window is a caption)
                own, earlier = 0, s * fr * 6
            else:
                f = (r - text) // ft
                own, earlier = ft, s * fr * 6 + f * 6
        else:
            own, earlier = fr * ft, s * fr * 6    # whole shot (its caption counted with the captions)
        want += 8 * text + own + min(topk, earlier) * ch
    assert n_pairs == want


def test_sparsity_of_eight_shot_shot_window_matches_paper():
    """The paper reports ~85 % of token pairs pruned for 8-shot scenes
    (Sec. 4, Table 1); the shot-window reading reproduces that from counts."""
    text, fr, ft, ch, S, k = 256, 9, 1560, 260, 8, 8
    N = S * (text + fr * ft)
    pairs = 0
    for s in range(S):
        earlier = s * fr * 6
        pairs += (text + fr * ft) * (S * text + fr * ft + min(k, earlier) * ch)
    sparsity = 1 - pairs / N ** 2
    assert 0.83 < sparsity < 0.87


@pytest.mark.parametrize("chunk", [10240, 5120, 2560, 1280])
def test_stream_layout_cuts_every_shot_on_its_own(chunk):
    """Fixed-size chunking of the flattened stream with shot-aligned boundaries (App. "Training
    Details"): no chunk crosses a shot or a caption boundary, only a shot's last chunk is short,
    and with the shot window the forced keys of a video query are its whole shot plus every caption."""
    lay = mi.config_layout("paper", chunk=chunk)
    lens = np.diff(lay.offsets)
    per_shot = 256 + 14040
    assert lay.N == 8 * per_shot and (lens > 0).all()
    for j in range(lay.C):
        s0, s1 = divmod(int(lay.offsets[j]), per_shot)[0], divmod(int(lay.offsets[j + 1]) - 1, per_shot)[0]
        assert s0 == s1 == lay.shot[j] == lay.window[j]
    video = np.ones(lay.C, bool)
    video[[np.searchsorted(lay.offsets, s) for s, _ in lay.text_spans]] = False
    tail = np.nonzero(video & (lens != chunk))[0]
    assert len(tail) == (8 if 14040 % chunk else 0) and (lens[tail] == 14040 % chunk).all()
    L = mo.OracleLayout.from_layout(lay)
    d = 4
    qidx = np.array([300, per_shot + 5000, 7 * per_shot + 14000], np.int32)
    q, k = _rand((1, 1, lay.N, d), 1), _rand((1, 1, lay.N, d), 2)
    sel, _ = mo.route(L, q, mo.pool(L, k), 5, True, qidx)
    per_video_chunks = -(-14040 // chunk)
    for r, i in enumerate(qidx):
        s = int(i) // per_shot
        got = sel[0, 0, r][sel[0, 0, r] >= 0]
        assert len(got) == min(5, s * per_video_chunks)            # candidates: video chunks of earlier shots
        assert (lay.shot[got] < s).all() and video[got].all()
    _, _, n_pairs = mo.attn_fwd(L, q, k, k, sel, None, qidx)
    want = sum(8 * 256 + 14040 + int(lens[sel[0, 0, r][sel[0, 0, r] >= 0]].sum()) for r in range(3))
    assert n_pairs == want
