"""Parity of moc_route_perturbed (Sec. 3.2, "Context Drop-off" / "Context Drop-in")
with the oracle: integer work, so rows must be identical. The only slack is the
routing tie rule: a row whose unperturbed selection (moc_route on the same
inputs) differs from the oracle's by a tolerated tie is not compared.
"""
import numpy as np
import pytest
import torch

import moc_inputs as mi
from oracle import moc_oracle as mo
from oracle import moc_perturb as mp
from paper_2508_21058_amd import binding as mb
from tests.test_gpu_parity import check_close, to_dev

pytestmark = pytest.mark.gpu


def _case(lay, H, d, topk, causal, p_max, lam, max_in, seed, dtype=torch.bfloat16, qidx=None, heads=None):
    N = lay.N
    q, k, _, _ = mi.qkv_do(1, H, N, d, seed, "cpu", bf16_round=True)
    qn, kn = q.numpy().astype(np.float64), k.numpy().astype(np.float64)
    L = mo.OracleLayout.from_layout(lay)
    meta = mb.chunk_meta(lay.offsets, lay.shot, lay.window, lay.text_spans)
    qd, kd = to_dev(q.numpy(), dtype), to_dev(k.numpy(), dtype)
    _, base = mb.route(meta, qd, kd, topk, causal)
    pooled, sel = mb.route_perturbed(meta, qd, kd, topk, causal, p_max, lam, max_in, seed)
    _, again = mb.route_perturbed(meta, qd, kd, topk, causal, p_max, lam, max_in, seed)
    torch.cuda.synchronize()
    assert torch.equal(sel, again)                       # same seed, same rows
    assert sel.shape == (1, H, N, topk + max_in)
    heads = list(range(H)) if heads is None else heads
    qi = np.arange(N) if qidx is None else np.asarray(qidx)
    kbar = mo.pool(L, kn[:, heads])
    base_ref, _ = mo.route(L, qn[:, heads], kbar, topk, causal, qi if qidx is not None else None)
    want = mp.perturb(L, base_ref, topk, causal, p_max, lam, max_in, seed, qidx=qi, heads=heads, H=H)
    got = sel.cpu().numpy()[:, heads][:, :, qi]
    base_gpu = base.cpu().numpy()[:, heads][:, :, qi] if topk > 0 else base_ref
    comparable = (base_gpu == base_ref).all(-1) if topk > 0 else np.ones(got.shape[:3], bool)
    assert (~comparable).sum() <= max(1, comparable.size // 1000)     # rows where routing itself hit a tolerated tie
    assert (got[comparable] == want[comparable]).all(), \
        f"{(got[comparable] != want[comparable]).any(-1).sum()} rows differ"
    meta.close()
    return got, want, L


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("causal", [True, False])
def test_random_ragged_layouts(seed, causal):
    lay = mi.random_layout(seed + 20, n_chunks=23, max_len=37, n_shots=3)
    _case(lay, H=3, d=64, topk=4, causal=causal, p_max=1.0, lam=1.5, max_in=5, seed=seed, dtype=torch.float32)


def test_regular_layout_bf16_many_text_chunks():
    lay = mi.multishot_layout(4, 16, 5, 64, 16, "frame")
    _case(lay, H=2, d=128, topk=6, causal=True, p_max=0.7, lam=2.0, max_in=8, seed=11)


def test_identity_when_both_regularisers_are_off():
    lay = mi.multishot_layout(2, 16, 4, 64, 32, "chunk")
    got, want, _ = _case(lay, H=2, d=64, topk=3, causal=True, p_max=0.0, lam=0.0, max_in=2, seed=5)
    assert (got[..., 3:] == -1).all()


def test_drop_in_only_topk_zero():
    lay = mi.multishot_layout(2, 8, 4, 32, 16, "frame")
    _case(lay, H=2, d=64, topk=0, causal=True, p_max=0.5, lam=3.0, max_in=6, seed=9)


def test_widest_row_and_more_draws_than_candidates():
    lay = mi.multishot_layout(3, 8, 3, 48, 8, "chunk")
    _case(lay, H=1, d=64, topk=16, causal=True, p_max=1.0, lam=12.0, max_in=16, seed=4)


def test_full_size_eight_shot_sampled_rows_and_properties():
    """The benchmark layout at full size: sampled rows of one head against the oracle, and properties on
    every row of that head: entries distinct, all of them candidates, -1 only at the end, and the number of
    added chunks close to lambda on average where enough candidates exist."""
    lay = mi.config_layout("eight")
    rng = np.random.default_rng(2)
    qidx = np.unique(np.concatenate([[0, 255, 256, 300, lay.N - 1], rng.choice(lay.N, 1500, replace=False)]))
    cfg = mi.CONFIGS["eight"]
    H, d, topk, lam, max_in = cfg["H"], cfg["d"], cfg["topk"], 1.0, 4
    q, k, _, _ = (t.to(torch.bfloat16).contiguous() if t is not None else None
                  for t in mi.qkv_do(1, H, lay.N, d, 1234, "cuda"))
    meta = mb.chunk_meta(lay.offsets, lay.shot, lay.window, lay.text_spans)
    _, base = mb.route(meta, q, k, topk, True)
    _, sel = mb.route_perturbed(meta, q, k, topk, True, 0.5, lam, max_in, 77)
    torch.cuda.synchronize()
    head = 13
    L = mo.OracleLayout.from_layout(lay)
    f64 = lambda t: t[0:1, head:head + 1].float().cpu().numpy().astype(np.float64)
    base_ref, _ = mo.route(L, f64(q), mo.pool(L, f64(k)), topk, True, qidx)
    want = mp.perturb(L, base_ref, topk, True, 0.5, lam, max_in, 77, qidx=qidx, heads=[head], H=H)[0, 0]
    got = sel[0, head].cpu().numpy()
    same_base = (base[0, head].cpu().numpy()[qidx] == base_ref[0, 0]).all(-1)
    assert same_base.mean() > 0.999 and (got[qidx][same_base] == want[same_base]).all()
    # properties on all N rows of the head
    valid = got >= 0
    assert (valid[:, :-1] >= valid[:, 1:]).all()                          # -1 only at the end
    srt = np.sort(np.where(valid, got, -np.arange(1, got.shape[1] + 1)), -1)
    assert (srt[:, 1:] != srt[:, :-1]).all()                              # no repeats
    cq = L.chunk_of[:, None]
    g = np.where(valid, got, 0)
    assert (~valid | ((g < cq) & (L.kind[g] == 0) & (L.win[g] != L.win[cq]))).all()
    base_np = base[0, head].cpu().numpy()
    n_added = (valid & ~(got[:, :, None] == base_np[:, None, :]).any(-1)).sum(-1)
    late = L.chunk_of > 100                                               # plenty of candidates
    mean_trunc = sum(min(j, max_in) * np.exp(-lam) * lam ** j / float(np.prod(np.arange(1, j + 1))) for j in range(40))
    assert abs(n_added[late].mean() - mean_trunc) < 0.01
    n_kept = (valid & (got[:, :, None] == base_np[:, None, :]).any(-1)).sum(-1)
    # floor(8 * U(0, 0.5)) is uniform on {0,1,2,3}: 1.5 removed on average
    assert abs((topk - n_kept[late]).mean() - 1.5) < 0.02
    meta.close()


def test_attention_accepts_the_wider_rows():
    """Forward and backward with the perturbed selection (width topk + max_in) against the oracle's
    attention on the oracle's perturbed selection."""
    lay = mi.multishot_layout(2, 24, 3, 96, 32, "frame")
    H, d, topk, max_in, seed = 2, 64, 2, 3, 21
    N = lay.N
    q, k, v, d_o = mi.qkv_do(1, H, N, d, seed, "cpu", bf16_round=True)
    qn, kn, vn, don = (t.numpy().astype(np.float64) for t in (q, k, v, d_o))
    L = mo.OracleLayout.from_layout(lay)
    base_ref, _ = mo.route(L, qn, mo.pool(L, kn), topk, True)
    sel_ref = mp.perturb(L, base_ref, topk, True, 1.0, 1.5, max_in, seed)
    o_ref, lse_ref, _ = mo.attn_fwd(L, qn, kn, vn, sel_ref)
    dq_ref = mo.attn_bwd_dq(L, qn, kn, vn, sel_ref, o_ref, lse_ref, don)
    dk_ref, dv_ref = mo.attn_bwd_dkdv(L, qn, kn, vn, sel_ref, o_ref, lse_ref, don)
    meta = mb.chunk_meta(lay.offsets, lay.shot, lay.window, lay.text_spans)
    qd, kd, vd, dod = (to_dev(t.numpy(), torch.bfloat16) for t in (q, k, v, d_o))
    _, sel = mb.route_perturbed(meta, qd, kd, topk, True, 1.0, 1.5, max_in, seed)
    torch.cuda.synchronize()
    assert (sel.cpu().numpy() == sel_ref).all()
    o, lse = mb.attn_fwd(meta, qd, kd, vd, sel)
    dq, dk, dv = mb.attn_bwd(meta, qd, kd, vd, o, lse, dod, sel)
    torch.cuda.synchronize()
    check_close("o", o.float().cpu().numpy(), o_ref)
    check_close("lse", lse.cpu().numpy(), lse_ref)
    check_close("dq", dq.float().cpu().numpy(), dq_ref)
    check_close("dk", dk.float().cpu().numpy(), dk_ref)
    check_close("dv", dv.float().cpu().numpy(), dv_ref)
    meta.close()


def test_bad_regulariser_arguments_are_refused():
    lay = mi.multishot_layout(1, 8, 2, 32, 16, "chunk")
    meta = mb.chunk_meta(lay.offsets, lay.shot, lay.window, lay.text_spans)
    q = torch.zeros(1, 1, lay.N, 64, dtype=torch.bfloat16, device="cuda")
    for kw in (dict(p_max=1.5), dict(p_max=-0.1), dict(lam=-1.0), dict(lam=float("inf")), dict(max_in=-1),
               dict(topk=20, max_in=13)):
        args = dict(topk=2, causal=True, p_max=0.5, lam=1.0, max_in=2, seed=1)
        args.update(kw)
        with pytest.raises(mb.MocError) as e:
            mb.route_perturbed(meta, q, q, args["topk"], args["causal"], args["p_max"], args["lam"], args["max_in"],
                               args["seed"])
        assert e.value.status == -2, kw
    meta.close()
