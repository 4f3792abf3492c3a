"""Thin ctypes binding of libmoc.so: argument marshalling only.

Every step of the layer runs inside the HIP library; torch is used for device
memory and for the current stream. The functions mirror the C entry points of
include/moc.h (moc_chunk_meta, moc_route, moc_attn_fwd, moc_attn_bwd).
There is no fallback: if the library is missing and cannot be built, loading
raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIBPATH = os.path.join(_HERE, "libmoc.so")
_lib = None

MOC_BF16, MOC_F32 = 0, 1
MOC_MAX_TOPK = 32

SYMBOLS = ["moc_status_string", "moc_last_error", "moc_chunk_meta", "moc_meta_destroy", "moc_meta_copy_tables",
           "moc_route_workspace_bytes", "moc_route", "moc_route_static", "moc_route_fused", "moc_route_fused_status", "moc_route_perturbed", "moc_outer_workspace_bytes", "moc_outer_route",
           "moc_outer_segments", "moc_reduce_layout", "moc_gather_rows", "moc_attn_workspace_bytes", "moc_attn_fwd",
           "moc_attn_bwd", "moc_attn_bwd_after_fwd",
           "moc_prof_enable", "moc_prof_read", "moc_probe"]


class MocError(RuntimeError):
    def __init__(self, status: int, where: str):
        l = lib()
        self.status = status
        msg = l.moc_status_string(status).decode()
        detail = l.moc_last_error().decode()
        super().__init__(f"{where}: {msg} ({status}): {detail}")


def lib():
    """Load libmoc.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIBPATH):
        from . import build as _build
        _build.build()
    l = C.CDLL(_LIBPATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    l.moc_status_string.restype = C.c_char_p
    l.moc_status_string.argtypes = [C.c_int]
    l.moc_last_error.restype = C.c_char_p
    l.moc_last_error.argtypes = []
    l.moc_chunk_meta.argtypes = [i32, i32, vp, vp, vp, vp, i32, vp, C.POINTER(vp)]
    l.moc_meta_destroy.argtypes = [vp]
    l.moc_meta_copy_tables.argtypes = [vp, vp, vp, vp]
    l.moc_route_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, C.c_int, C.POINTER(sz)]
    l.moc_route.argtypes = [vp, i32, i32, i32, C.c_int, vp, vp, i32, i32, vp, vp, vp, sz, vp]
    l.moc_route_fused.argtypes = l.moc_route.argtypes
    l.moc_route_fused_status.argtypes = [C.POINTER(i32)]
    l.moc_route_static.argtypes = [vp, i32, i32, i32, C.c_int, vp, vp, i32, i32, vp, vp, vp]
    l.moc_attn_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, C.c_int, C.c_int, C.POINTER(sz)]
    l.moc_attn_fwd.argtypes = [vp, i32, i32, i32, C.c_int, vp, vp, vp, vp, i32, C.c_float, vp, vp, vp, sz, vp]
    l.moc_attn_bwd.argtypes = [vp, i32, i32, i32, C.c_int, vp, vp, vp, vp, vp, vp, vp, i32, C.c_float,
                               vp, vp, vp, vp, sz, vp]
    l.moc_attn_bwd_after_fwd.argtypes = l.moc_attn_bwd.argtypes
    l.moc_outer_segments.argtypes = [i32, vp, vp, vp, i32, vp, vp, C.POINTER(i32)]
    l.moc_reduce_layout.argtypes = [i32, vp, vp, vp, vp, i32, i32, vp, i32, vp, vp, vp, vp, vp, C.POINTER(i32),
                                    C.POINTER(i32), vp]
    l.moc_route_perturbed.argtypes = [vp, i32, i32, i32, C.c_int, vp, vp, i32, i32, C.c_float, C.c_float, i32,
                                      C.c_uint64, vp, vp, vp, sz, vp]
    l.moc_outer_workspace_bytes.argtypes = [i32, i32, i32, C.POINTER(sz)]
    l.moc_outer_route.argtypes = [i32, i32, C.c_int, vp, i32, vp, vp, i32, i32, i32, vp, vp, vp, vp, C.POINTER(i32),
                                  vp, sz, vp]
    l.moc_gather_rows.argtypes = [i32, i32, i32, vp, i32, vp, vp, vp, sz, vp]
    l.moc_probe.argtypes = [i32, vp, sz, i32, vp, C.POINTER(C.c_float), C.POINTER(C.c_double)]
    l.moc_prof_enable.argtypes = [C.c_int]
    l.moc_prof_read.argtypes = [i32, C.c_char_p, sz, C.POINTER(i32), C.POINTER(C.c_float)]
    for name in SYMBOLS:
        if name not in ("moc_status_string", "moc_last_error"):
            getattr(l, name).restype = C.c_int
    _lib = l
    return l


def _check(rc: int, where: str):
    if rc != 0:
        raise MocError(rc, where)


def _stream():
    """Current torch stream handle; None (the default stream) when no GPU is
    present, so that argument validation can be exercised on a CPU-only host."""
    if not torch.cuda.is_available():
        return None
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return MOC_BF16
    if t.dtype == torch.float32:
        return MOC_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


class Meta:
    """Owner of a moc_meta handle (stage a)."""

    def __init__(self, handle, N, C_, T):
        self.handle, self.N, self.C, self.T = handle, N, C_, T

    def tables(self):
        """Device tables copied back: (chunk_of [N], chunk_kind [C], chunk_window [C])."""
        cof = np.zeros(self.N, np.int32)
        kind = np.zeros(self.C, np.int32)
        win = np.zeros(self.C, np.int32)
        _check(lib().moc_meta_copy_tables(self.handle, cof.ctypes.data, kind.ctypes.data, win.ctypes.data),
               "moc_meta_copy_tables")
        return cof, kind, win

    def close(self):
        if self.handle:
            lib().moc_meta_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def chunk_meta(offsets, shot, window=None, text_spans=None) -> Meta:
    off, sh = _i32(offsets), _i32(shot)
    win = None if window is None else _i32(window)
    spans = _i32(text_spans).reshape(-1, 2) if text_spans is not None else np.zeros((0, 2), np.int32)
    Cn, N, T = off.shape[0] - 1, int(off[-1]) if off.size else 0, spans.shape[0]
    h = C.c_void_p()
    rc = lib().moc_chunk_meta(N, Cn, off.ctypes.data, sh.ctypes.data, None if win is None else win.ctypes.data,
                              spans.ctypes.data if T else None, T, _stream(), C.byref(h))
    _check(rc, "moc_chunk_meta")
    return Meta(h, N, Cn, T)


def _shape(meta: Meta, q: torch.Tensor):
    B, H, N, d = q.shape
    if N != meta.N:
        raise ValueError(f"tensor has N={N}, layout has N={meta.N}")
    return B, H, N, d


def _need_contig(*ts):
    for t in ts:
        if t is not None and not (t.is_cuda and t.is_contiguous()):
            raise ValueError("tensors must be contiguous CUDA tensors")


def route(meta: Meta, q: torch.Tensor, k: torch.Tensor, topk: int, causal: bool = True
          ) -> Tuple[torch.Tensor, torch.Tensor]:
    """-> pooled_k [B,H,C,d] fp32, sel [B,H,N,topk] int32."""
    B, H, N, d = _shape(meta, q)
    _need_contig(q, k)
    dt = _dtype_code(q)
    nbytes = C.c_size_t()
    _check(lib().moc_route_workspace_bytes(meta.handle, B, H, d, topk, dt, C.byref(nbytes)),
           "moc_route_workspace_bytes")
    ws = torch.empty(max(nbytes.value, 16), dtype=torch.uint8, device=q.device)
    pooled = torch.empty(B, H, meta.C, d, dtype=torch.float32, device=q.device)
    sel = torch.empty(B, H, N, max(topk, 0), dtype=torch.int32, device=q.device)
    _check(lib().moc_route(meta.handle, B, H, d, dt, _ptr(q), _ptr(k), topk, int(bool(causal)), _ptr(pooled),
                           _ptr(sel) if topk > 0 else None, _ptr(ws), nbytes.value, _stream()), "moc_route")
    return pooled, sel


def route_fused(meta: Meta, q: torch.Tensor, k: torch.Tensor, topk: int, causal: bool = True):
    """moc_route_fused: pooling, scoring and top-k in one launch -> pooled_k, sel (as route)."""
    B, H, N, d = _shape(meta, q)
    _need_contig(q, k)
    dt = _dtype_code(q)
    nbytes = C.c_size_t()
    _check(lib().moc_route_workspace_bytes(meta.handle, B, H, d, topk, dt, C.byref(nbytes)),
           "moc_route_workspace_bytes")
    ws = torch.empty(max(nbytes.value, 16), dtype=torch.uint8, device=q.device)
    pooled = torch.empty(B, H, meta.C, d, dtype=torch.float32, device=q.device)
    sel = torch.empty(B, H, N, max(topk, 0), dtype=torch.int32, device=q.device)
    _check(lib().moc_route_fused(meta.handle, B, H, d, dt, _ptr(q), _ptr(k), topk, int(bool(causal)), _ptr(pooled),
                                 _ptr(sel), _ptr(ws), nbytes.value, _stream()), "moc_route_fused")
    return pooled, sel


def route_fused_timed_out() -> bool:
    t = C.c_int32()
    _check(lib().moc_route_fused_status(C.byref(t)), "moc_route_fused_status")
    return bool(t.value)


def route_static(meta: Meta, q: torch.Tensor, k: torch.Tensor, topk: int, causal: bool = True, out=None):
    """moc_route_static: routing with the library's static scratch. `out` = (pooled_k, sel) tensors to fill
    (the call itself allocates nothing; without `out` this wrapper allocates the two outputs)."""
    B, H, N, d = _shape(meta, q)
    _need_contig(q, k)
    pooled, sel = out if out is not None else (
        torch.empty(B, H, meta.C, d, dtype=torch.float32, device=q.device),
        torch.empty(B, H, N, max(topk, 0), dtype=torch.int32, device=q.device))
    _check(lib().moc_route_static(meta.handle, B, H, d, _dtype_code(q), _ptr(q), _ptr(k), topk, int(bool(causal)),
                                  _ptr(pooled), _ptr(sel) if topk > 0 else None, _stream()), "moc_route_static")
    return pooled, sel


def route_perturbed(meta: Meta, q: torch.Tensor, k: torch.Tensor, topk: int, causal: bool, p_max: float,
                    lam: float, max_in: int, seed: int) -> Tuple[torch.Tensor, torch.Tensor]:
    """Routing with context drop-off and drop-in -> pooled_k [B,H,C,d] fp32, sel [B,H,N,topk+max_in] int32."""
    B, H, N, d = _shape(meta, q)
    _need_contig(q, k)
    dt = _dtype_code(q)
    nbytes = C.c_size_t()
    _check(lib().moc_route_workspace_bytes(meta.handle, B, H, d, topk, dt, C.byref(nbytes)),
           "moc_route_workspace_bytes")
    ws = torch.empty(max(nbytes.value, 16), dtype=torch.uint8, device=q.device)
    pooled = torch.empty(B, H, meta.C, d, dtype=torch.float32, device=q.device)
    width = max(topk + max_in, 0)
    sel = torch.empty(B, H, N, width, dtype=torch.int32, device=q.device)
    _check(lib().moc_route_perturbed(meta.handle, B, H, d, dt, _ptr(q), _ptr(k), int(topk), int(bool(causal)),
                                     float(p_max), float(lam), int(max_in), int(seed), _ptr(pooled),
                                     _ptr(sel) if width > 0 else None, _ptr(ws), nbytes.value, _stream()),
           "moc_route_perturbed")
    return pooled, sel


def attn_workspace(meta: Meta, B: int, H: int, d: int, topk: int, dtype: torch.dtype, with_bwd: bool,
                   device="cuda") -> torch.Tensor:
    dt = MOC_BF16 if dtype == torch.bfloat16 else MOC_F32
    nbytes = C.c_size_t()
    _check(lib().moc_attn_workspace_bytes(meta.handle, B, H, d, topk, dt, int(with_bwd), C.byref(nbytes)),
           "moc_attn_workspace_bytes")
    return torch.empty(max(nbytes.value, 16), dtype=torch.uint8, device=device)


def attn_fwd(meta: Meta, q, k, v, sel, scale: Optional[float] = None, workspace: Optional[torch.Tensor] = None,
             out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None):
    """-> o [B,H,N,d] (dtype of q), lse [B,H,N] fp32."""
    B, H, N, d = _shape(meta, q)
    _need_contig(q, k, v, sel)
    topk = int(sel.shape[-1])
    scale = float(d ** -0.5 if scale is None else scale)
    ws = workspace if workspace is not None else attn_workspace(meta, B, H, d, topk, q.dtype, False, q.device)
    o, lse = out if out is not None else (torch.empty_like(q),
                                          torch.empty(B, H, N, dtype=torch.float32, device=q.device))
    _check(lib().moc_attn_fwd(meta.handle, B, H, d, _dtype_code(q), _ptr(q), _ptr(k), _ptr(v),
                              _ptr(sel) if topk > 0 else None, topk, scale, _ptr(o), _ptr(lse), _ptr(ws),
                              ws.numel(), _stream()), "moc_attn_fwd")
    return o, lse


def attn_bwd(meta: Meta, q, k, v, o, lse, d_o, sel, scale: Optional[float] = None,
             workspace: Optional[torch.Tensor] = None, out=None, after_fwd: bool = False):
    """-> dq, dk, dv [B,H,N,d] (dtype of q). after_fwd: call moc_attn_bwd_after_fwd (the lists the
    forward left in `workspace` are reused)."""
    B, H, N, d = _shape(meta, q)
    _need_contig(q, k, v, o, lse, d_o, sel)
    topk = int(sel.shape[-1])
    scale = float(d ** -0.5 if scale is None else scale)
    ws = workspace if workspace is not None else attn_workspace(meta, B, H, d, topk, q.dtype, True, q.device)
    dq, dk, dv = out if out is not None else (torch.empty_like(q), torch.empty_like(q), torch.empty_like(q))
    fn = lib().moc_attn_bwd_after_fwd if after_fwd else lib().moc_attn_bwd
    _check(fn(meta.handle, B, H, d, _dtype_code(q), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse),
              _ptr(d_o), _ptr(sel) if topk > 0 else None, topk, scale, _ptr(dq), _ptr(dk), _ptr(dv),
              _ptr(ws), ws.numel(), _stream()), "moc_attn_bwd")
    return dq, dk, dv


def prof_enable(on: bool):
    _check(lib().moc_prof_enable(int(on)), "moc_prof_enable")


def prof_read():
    """-> {kernel name: (launches, total_ms)} for the launches recorded since prof_enable(True)."""
    n = lib().moc_prof_read(-1, None, 0, None, None)
    if n < 0:
        raise MocError(n, "moc_prof_read")
    out = {}
    for i in range(n):
        buf = C.create_string_buffer(128)
        cnt, ms = C.c_int32(), C.c_float()
        _check(lib().moc_prof_read(i, buf, 128, C.byref(cnt), C.byref(ms)), "moc_prof_read")
        out[buf.value.decode()] = (cnt.value, ms.value)
    return out


_PROBE_KINDS = {"copy": 0, "mfma": 1, "mfma4": 2, "valu4": 3, "mfma4+valu4": 4, "mfma4+valu_same_wave": 5,
                "lds_read": 6, "lds_read_transposed": 7, "copy_to_lds_async": 8, "copy_via_registers": 9}


def probe(kind: str, buf: torch.Tensor, iters: int):
    """Machine probe: kind 'copy' streams the first half of `buf` into the second, 'mfma' runs
    a loop of independent bf16 MFMA chains. -> (milliseconds, bytes moved or flops issued)."""
    assert buf.is_cuda and buf.is_contiguous()
    ms, units = C.c_float(), C.c_double()
    _check(lib().moc_probe(_PROBE_KINDS[kind], _ptr(buf), buf.numel() * buf.element_size(),
                           int(iters), _stream(), C.byref(ms), C.byref(units)), "moc_probe")
    return ms.value, units.value



def outer_route(x: torch.Tensor, seg_offsets, mandatory, g: int, M: int, causal: bool = True):
    """Outer-loop routing over features x [N, D] -> seg_mean [P, D] fp32, scores [P] fp32 (device),
    selected [M] (numpy, best first, -1 padded), kept (ascending list of segments of the reduced stream)."""
    assert x.is_cuda and x.dim() == 2
    _need_contig(x)
    N, D = x.shape
    off = np.ascontiguousarray(seg_offsets, dtype=np.int32)
    P = off.shape[0] - 1
    mand = None if mandatory is None else np.ascontiguousarray(mandatory, dtype=np.int32)
    nbytes = C.c_size_t()
    _check(lib().moc_outer_workspace_bytes(N, D, P, C.byref(nbytes)), "moc_outer_workspace_bytes")
    ws = torch.empty(max(nbytes.value, 16), dtype=torch.uint8, device=x.device)
    mean = torch.empty(P, D, dtype=torch.float32, device=x.device)
    scores = torch.empty(P, dtype=torch.float32, device=x.device)
    selected = np.full(max(M, 1), -1, dtype=np.int32)
    kept = np.zeros(P, dtype=np.int32)
    n_kept = C.c_int32()
    _check(lib().moc_outer_route(N, D, _dtype_code(x), _ptr(x), P, off.ctypes.data,
                                 None if mand is None else mand.ctypes.data, int(g), int(M), int(bool(causal)),
                                 _ptr(mean), _ptr(scores), selected.ctypes.data, kept.ctypes.data, C.byref(n_kept),
                                 _ptr(ws), nbytes.value, _stream()), "moc_outer_route")
    return mean, scores, selected[:max(M, 0)], kept[:n_kept.value].tolist()


def gather_rows(src: torch.Tensor, ranges) -> torch.Tensor:
    """src [..., N, d] (contiguous) -> [..., sum of lengths, d]: the rows of the listed (start, length) ranges."""
    assert src.is_cuda and src.dim() >= 2
    _need_contig(src)
    rg = np.ascontiguousarray(ranges, dtype=np.int32).reshape(-1, 2)
    n_src, dlast = src.shape[-2], src.shape[-1]
    outer = int(np.prod(src.shape[:-2])) if src.dim() > 2 else 1
    n_dst = int(rg[:, 1].sum())
    dst = torch.empty(*src.shape[:-2], n_dst, dlast, dtype=src.dtype, device=src.device)
    ws = torch.empty(max(16 * rg.shape[0], 16), dtype=torch.uint8, device=src.device)
    _check(lib().moc_gather_rows(outer, n_src, dlast * src.element_size(), _ptr(src), rg.shape[0], rg.ctypes.data,
                                 _ptr(dst), _ptr(ws), ws.numel(), _stream()), "moc_gather_rows")
    return dst


def outer_segments(offsets, shot, text_spans):
    """Segments of the outer loop -> (seg_offsets [P+1], is_caption [P]) as numpy int32."""
    off, sh = _i32(offsets), _i32(shot)
    spans = _i32(text_spans).reshape(-1, 2) if text_spans is not None else np.zeros((0, 2), np.int32)
    Cn, T = off.shape[0] - 1, spans.shape[0]
    seg = np.zeros(Cn + 1, np.int32)
    cap = np.zeros(Cn, np.int32)
    P = C.c_int32()
    _check(lib().moc_outer_segments(Cn, off.ctypes.data, sh.ctypes.data, spans.ctypes.data if T else None, T,
                                    seg.ctypes.data, cap.ctypes.data, C.byref(P)), "moc_outer_segments")
    return seg[:P.value + 1].copy(), cap[:P.value].copy()


def reduce_layout(offsets, shot, window, text_spans, seg_offsets, kept):
    """Layout of the reduced stream -> (offsets, shot, window, text_spans [T,2], ranges [n_kept,2])."""
    off, sh = _i32(offsets), _i32(shot)
    win = None if window is None else _i32(window)
    spans = _i32(text_spans).reshape(-1, 2) if text_spans is not None else np.zeros((0, 2), np.int32)
    seg, kp = _i32(seg_offsets), _i32(kept)
    Cn, T, P = off.shape[0] - 1, spans.shape[0], seg.shape[0] - 1
    o_off, o_shot, o_win = np.zeros(Cn + 1, np.int32), np.zeros(Cn, np.int32), np.zeros(Cn, np.int32)
    o_spans = np.zeros((T + len(kp) + 1, 2), np.int32)     # a span cut by segment boundaries gives several pieces
    ranges = np.zeros((max(len(kp), 1), 2), np.int32)
    oC, oT = C.c_int32(), C.c_int32()
    _check(lib().moc_reduce_layout(Cn, off.ctypes.data, sh.ctypes.data, None if win is None else win.ctypes.data,
                                   spans.ctypes.data if T else None, T, P, seg.ctypes.data, len(kp), kp.ctypes.data,
                                   o_off.ctypes.data, o_shot.ctypes.data, o_win.ctypes.data, o_spans.ctypes.data,
                                   C.byref(oC), C.byref(oT), ranges.ctypes.data), "moc_reduce_layout")
    return (o_off[:oC.value + 1].copy(), o_shot[:oC.value].copy(), o_win[:oC.value].copy(),
            o_spans[:oT.value].copy(), ranges[:len(kp)].copy())
