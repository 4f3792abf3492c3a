"""ctypes wrapper around the C oracle (oracle/moc_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu-baseline leg. Nothing in the product package imports it.

All tensors are numpy arrays; heads are looped here, one (batch, head) slice
per C call, converted to float64 on the way in.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moc_oracle.c")
_LIB = os.path.join(_HERE, "libmoc_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_ip = C.POINTER(C.c_int)
_dp = C.POINTER(C.c_double)
_lp = C.POINTER(C.c_longlong)


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        for name in ("moc_oracle_chunk_map", "moc_oracle_chunk_kind", "moc_oracle_pool",
                     "moc_oracle_route", "moc_oracle_attn_fwd", "moc_oracle_attn_bwd_dq",
                     "moc_oracle_attn_bwd_dkdv"):
            getattr(_lib, name).restype = None
    return _lib


def _i(a):
    return None if a is None else a.ctypes.data_as(_ip)


def _d(a):
    return None if a is None else a.ctypes.data_as(_dp)


def _ci(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _cd(a):
    return np.ascontiguousarray(a, dtype=np.float64)


class OracleLayout:
    """Chunk tables derived by the oracle's own step O1."""

    def __init__(self, offsets, window=None, text_spans=None):
        self.off = _ci(offsets)
        self.C = int(self.off.shape[0] - 1)
        self.N = int(self.off[-1])
        self.win = _ci(window) if window is not None else np.arange(self.C, dtype=np.int32)
        spans = _ci(text_spans).reshape(-1, 2) if text_spans is not None else np.zeros((0, 2), np.int32)
        self.spans = spans
        self.kind = np.zeros(self.C, dtype=np.int32)
        lib().moc_oracle_chunk_kind(self.C, _i(self.off), int(spans.shape[0]), _i(spans), _i(self.kind))
        self.chunk_of = np.zeros(self.N, dtype=np.int32)
        lib().moc_oracle_chunk_map(self.N, self.C, _i(self.off), _i(self.chunk_of))

    @classmethod
    def from_layout(cls, lay):
        return cls(lay.offsets, lay.window, lay.text_spans)


def pool(L: OracleLayout, k: np.ndarray) -> np.ndarray:
    """k [B,H,N,d] -> mean-pooled keys [B,H,C,d] (float64)."""
    B, H, N, d = k.shape
    out = np.zeros((B, H, L.C, d), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            kk = _cd(k[b, h])
            lib().moc_oracle_pool(N, d, L.C, _i(L.off), _d(kk), _d(out[b, h]))
    return out


def route(L: OracleLayout, q: np.ndarray, kbar: np.ndarray, topk: int, causal: bool = True,
          qidx: Optional[Sequence[int]] = None, want_scores: bool = False):
    """q [B,H,N,d], kbar [B,H,C,d] -> sel [B,H,nq,topk] int32 (+ scores [B,H,nq,C], eligible count)."""
    B, H, N, d = q.shape
    qi = _ci(qidx) if qidx is not None else None
    nq = N if qi is None else int(qi.shape[0])
    sel = np.full((B, H, nq, max(topk, 0)), -1, dtype=np.int32)
    scores = np.zeros((B, H, nq, L.C), dtype=np.float64) if want_scores else None
    total = 0
    for b in range(B):
        for h in range(H):
            qq, kb = _cd(q[b, h]), _cd(kbar[b, h])
            ne = C.c_longlong(0)
            s = np.zeros((nq, max(topk, 1)), dtype=np.int32)
            lib().moc_oracle_route(N, d, L.C, _i(L.off), _i(L.kind), _i(L.win), int(bool(causal)), int(topk),
                                   _d(qq), _d(kb), nq, _i(qi), _i(s),
                                   _d(scores[b, h]) if want_scores else None, C.byref(ne))
            if topk > 0:
                sel[b, h] = s[:, :topk]
            total += ne.value
    return (sel, scores, total) if want_scores else (sel, total)


def attn_fwd(L: OracleLayout, q, k, v, sel, scale: Optional[float] = None,
             qidx: Optional[Sequence[int]] = None):
    """-> o [B,H,nq,d], lse [B,H,nq] (float64), n_pairs. sel [B,H,nq,topk]."""
    B, H, N, d = q.shape
    scale = float(scale if scale is not None else d ** -0.5)
    qi = _ci(qidx) if qidx is not None else None
    nq = N if qi is None else int(qi.shape[0])
    topk = int(sel.shape[-1])
    o = np.zeros((B, H, nq, d), dtype=np.float64)
    lse = np.zeros((B, H, nq), dtype=np.float64)
    total = 0
    for b in range(B):
        for h in range(H):
            qq, kk, vv = _cd(q[b, h]), _cd(k[b, h]), _cd(v[b, h])
            s = _ci(sel[b, h]).reshape(nq, topk) if topk > 0 else np.zeros((nq, 1), np.int32)
            npairs = C.c_longlong(0)
            lib().moc_oracle_attn_fwd(N, d, L.C, _i(L.off), _i(L.kind), _i(L.win), topk, _i(s),
                                      _d(qq), _d(kk), _d(vv), C.c_double(scale), nq, _i(qi),
                                      _d(o[b, h]), _d(lse[b, h]), C.byref(npairs))
            total += npairs.value
    return o, lse, total


def attn_bwd_dq(L: OracleLayout, q, k, v, sel, o, lse, d_o, scale: Optional[float] = None,
                qidx: Optional[Sequence[int]] = None):
    """dq [B,H,nq,d]; o, lse, d_o, sel are indexed like the query list."""
    B, H, N, d = q.shape
    scale = float(scale if scale is not None else d ** -0.5)
    qi = _ci(qidx) if qidx is not None else None
    nq = N if qi is None else int(qi.shape[0])
    topk = int(sel.shape[-1])
    dq = np.zeros((B, H, nq, d), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            qq, kk, vv = _cd(q[b, h]), _cd(k[b, h]), _cd(v[b, h])
            oo, ll, dd = _cd(o[b, h]), _cd(lse[b, h]), _cd(d_o[b, h])
            s = _ci(sel[b, h]).reshape(nq, topk) if topk > 0 else np.zeros((nq, 1), np.int32)
            lib().moc_oracle_attn_bwd_dq(N, d, L.C, _i(L.off), _i(L.kind), _i(L.win), topk, _i(s),
                                         _d(qq), _d(kk), _d(vv), C.c_double(scale), nq, _i(qi),
                                         _d(oo), _d(ll), _d(dd), _d(dq[b, h]))
    return dq


def attn_bwd_dkdv(L: OracleLayout, q, k, v, sel, o, lse, d_o, scale: Optional[float] = None,
                  chunks: Optional[Sequence[int]] = None):
    """dk, dv [B,H,N,d]; rows outside the listed chunks stay zero. sel/o/lse/d_o cover all N queries."""
    B, H, N, d = q.shape
    scale = float(scale if scale is not None else d ** -0.5)
    ch = _ci(chunks) if chunks is not None else None
    nch = L.C if ch is None else int(ch.shape[0])
    topk = int(sel.shape[-1])
    dk = np.zeros((B, H, N, d), dtype=np.float64)
    dv = np.zeros((B, H, N, d), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            qq, kk, vv = _cd(q[b, h]), _cd(k[b, h]), _cd(v[b, h])
            oo, ll, dd = _cd(o[b, h]), _cd(lse[b, h]), _cd(d_o[b, h])
            s = _ci(sel[b, h]).reshape(N, topk) if topk > 0 else np.zeros((N, 1), np.int32)
            lib().moc_oracle_attn_bwd_dkdv(N, d, L.C, _i(L.off), _i(L.kind), _i(L.win), topk, _i(s),
                                           _d(qq), _d(kk), _d(vv), C.c_double(scale),
                                           _d(oo), _d(ll), _d(dd), nch, _i(ch), _d(dk[b, h]), _d(dv[b, h]))
    return dk, dv


def moc_layer(L: OracleLayout, q, k, v, topk: int, causal: bool = True, d_o=None,
              scale: Optional[float] = None):
    """Whole layer on all queries: pool -> route -> attention (-> backward)."""
    kbar = pool(L, k)
    sel, n_el = route(L, q, kbar, topk, causal)
    o, lse, n_pairs = attn_fwd(L, q, k, v, sel, scale)
    out = dict(kbar=kbar, sel=sel, o=o, lse=lse, n_eligible=n_el, n_pairs=n_pairs)
    if d_o is not None:
        out["dq"] = attn_bwd_dq(L, q, k, v, sel, o, lse, d_o, scale)
        out["dk"], out["dv"] = attn_bwd_dkdv(L, q, k, v, sel, o, lse, d_o, scale)
    return out
