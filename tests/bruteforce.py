"""Brute-force checker for the MoC layer, written separately from the oracle.

It builds the full [N, C] score matrix, sets masked entries to -inf, selects by
k repeated arg-max passes (no sort), expands the choice to an explicit N x N
boolean mask and runs dense masked softmax attention (Sec. 3.1 Eq. 1 with a
mask). Gradients come from torch autograd on that dense masked attention.
Only usable for small N.
"""
import numpy as np
import torch


def chunk_tables(lay):
    off = np.asarray(lay.offsets, dtype=np.int64)
    C = off.shape[0] - 1
    N = int(off[-1])
    chunk_of = np.searchsorted(off, np.arange(N), side="right") - 1
    is_text = np.zeros(C, dtype=bool)
    for (s, e) in np.asarray(lay.text_spans).reshape(-1, 2):
        is_text |= (off[:-1] >= s) & (off[1:] <= e)
    win = np.asarray(lay.window, dtype=np.int64) if lay.window is not None else np.arange(C)
    return off, C, N, chunk_of, is_text, win


def mandatory_matrix(lay):
    """[N, C] bool: chunk j is a forced link of query i (all text + own window)."""
    off, C, N, chunk_of, is_text, win = chunk_tables(lay)
    return is_text[None, :] | (win[None, :] == win[chunk_of][:, None])


def select(lay, q, k, topk, causal=True):
    """q, k [N, d] float64 -> (sel [N, topk] int, scores [N, C] with -inf at masked, kbar)."""
    off, C, N, chunk_of, is_text, win = chunk_tables(lay)
    kbar = np.stack([k[off[j]:off[j + 1]].mean(axis=0) for j in range(C)])
    scores = q @ kbar.T
    masked = mandatory_matrix(lay).copy()
    if causal:
        masked |= np.arange(C)[None, :] >= chunk_of[:, None]
    scores = np.where(masked, -np.inf, scores)
    work = scores.copy()
    sel = np.full((N, topk), -1, dtype=np.int64)
    rows = np.arange(N)
    for r in range(topk):
        best = np.argmax(work, axis=1)          # first maximum = lowest index on ties
        ok = np.isfinite(work[rows, best])
        sel[ok, r] = best[ok]
        work[rows[ok], best[ok]] = -np.inf
    return sel, scores, kbar


def token_mask(lay, sel):
    """[N, N] bool: query i attends token t."""
    off, C, N, chunk_of, is_text, win = chunk_tables(lay)
    cm = mandatory_matrix(lay).copy()
    rows = np.arange(N)
    for r in range(sel.shape[1]):
        ok = sel[:, r] >= 0
        cm[rows[ok], sel[ok, r]] = True
    return cm[:, chunk_of]


def dense_masked_attention(q, k, v, mask, d_o=None, scale=None):
    """float64 dense softmax attention with a boolean mask; autograd for gradients."""
    qt = torch.tensor(q, dtype=torch.float64, requires_grad=d_o is not None)
    kt = torch.tensor(k, dtype=torch.float64, requires_grad=d_o is not None)
    vt = torch.tensor(v, dtype=torch.float64, requires_grad=d_o is not None)
    m = torch.tensor(mask)
    scale = scale if scale is not None else q.shape[-1] ** -0.5
    logits = (qt @ kt.T) * scale
    logits = logits.masked_fill(~m, float("-inf"))
    lse = torch.logsumexp(logits, dim=-1)
    o = torch.softmax(logits, dim=-1) @ vt
    out = dict(o=o.detach().numpy(), lse=lse.detach().numpy())
    if d_o is not None:
        o.backward(torch.tensor(d_o, dtype=torch.float64))
        out.update(dq=qt.grad.numpy(), dk=kt.grad.numpy(), dv=vt.grad.numpy())
    return out


def moc_bruteforce(lay, q, k, v, topk, causal=True, d_o=None):
    sel, scores, kbar = select(lay, q, k, topk, causal)
    mask = token_mask(lay, sel)
    out = dense_masked_attention(q, k, v, mask, d_o)
    out.update(sel=sel, scores=scores, kbar=kbar, mask=mask)
    return out
