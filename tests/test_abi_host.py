"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/moc.h declares, and rejects bad layouts before any device
work."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import moc_inputs as mi
from paper_2508_21058_amd import binding as mb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "moc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moc_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = mb.lib()
    names = _declared_symbols()
    assert {"moc_chunk_meta", "moc_route", "moc_attn_fwd", "moc_attn_bwd"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(mb.SYMBOLS) == names


def test_status_strings():
    lib = mb.lib()
    assert lib.moc_status_string(0) == b"ok"
    for code in range(-10, 0):
        assert lib.moc_status_string(code) != b"unknown status"


def _meta_rc(off, shot, win, spans):
    lib = mb.lib()
    off = np.ascontiguousarray(off, np.int32)
    shot = np.ascontiguousarray(shot, np.int32)
    win = None if win is None else np.ascontiguousarray(win, np.int32)
    spans = np.ascontiguousarray(spans, np.int32).reshape(-1, 2)
    h = C.c_void_p()
    rc = lib.moc_chunk_meta(int(off[-1]), off.shape[0] - 1, off.ctypes.data, shot.ctypes.data,
                            None if win is None else win.ctypes.data,
                            spans.ctypes.data if spans.size else None, spans.shape[0], None, C.byref(h))
    assert h.value is None or rc == 0
    return rc


@pytest.mark.parametrize("case,want", [
    (dict(off=[0, 4, 4, 9], shot=[0, 0, 0], win=None, spans=[]), -3),          # not strictly increasing
    (dict(off=[1, 4, 9], shot=[0, 0], win=None, spans=[]), -3),                # does not start at 0
    (dict(off=[0, 4, 9], shot=[1, 0], win=None, spans=[]), -10),               # shot decreases
    (dict(off=[0, 4, 9], shot=[0, 0], win=None, spans=[[0, 3]]), -4),          # span not chunk aligned
    (dict(off=[0, 4, 9], shot=[0, 0], win=None, spans=[[4, 4]]), -4),          # empty span
    (dict(off=[0, 4, 9], shot=[0, 0], win=None, spans=[[4, 9], [0, 4]]), -4),  # unsorted spans
    (dict(off=[0, 4, 9, 12], shot=[0, 0, 0], win=[7, 8, 7], spans=[]), -5),    # window id not contiguous
    (dict(off=[0, 4, 9], shot=[0, 1], win=[3, 3], spans=[]), -5),              # window spans two shots
])
def test_bad_layouts_are_rejected_before_device_work(case, want):
    assert _meta_rc(**case) == want
    assert mb.lib().moc_last_error() != b""


def test_null_and_shape_errors():
    lib = mb.lib()
    h = C.c_void_p()
    off = np.array([0, 4], np.int32)
    shot = np.array([0], np.int32)
    assert lib.moc_chunk_meta(4, 1, None, shot.ctypes.data, None, None, 0, None, C.byref(h)) == -1
    assert lib.moc_chunk_meta(0, 0, off.ctypes.data, shot.ctypes.data, None, None, 0, None, C.byref(h)) == -2
    n = C.c_size_t()
    assert lib.moc_attn_workspace_bytes(None, 1, 1, 128, 4, 0, 0, C.byref(n)) == -1
    assert lib.moc_route(None, 1, 1, 128, 0, None, None, 4, 1, None, None, None, 0, None) == -1
    assert lib.moc_attn_fwd(None, 1, 1, 128, 0, None, None, None, None, 4, 0.1, None, None, None, 0, None) == -1


def test_probe_rejects_bad_arguments_before_any_launch():
    lib = mb.lib()
    ms, units = C.c_float(), C.c_double()
    assert lib.moc_probe(0, None, C.c_size_t(64), 1, None, C.byref(ms), C.byref(units)) == -1
    fake = C.c_void_p(0x1000)                       # never dereferenced: every call below is rejected on the host
    assert lib.moc_probe(10, fake, C.c_size_t(64), 1, None, C.byref(ms), C.byref(units)) == -2
    assert lib.moc_probe(8, fake, C.c_size_t(600000), 1, None, C.byref(ms), C.byref(units)) == -7   # needs 1 MiB
    assert lib.moc_probe(4, fake, C.c_size_t(4096), 1, None, C.byref(ms), C.byref(units)) == -7
    assert lib.moc_probe(0, fake, C.c_size_t(64), 0, None, C.byref(ms), C.byref(units)) == -2
    assert lib.moc_probe(0, C.c_void_p(0x1004), C.c_size_t(64), 1, None, C.byref(ms), C.byref(units)) == -8
    assert lib.moc_probe(0, fake, C.c_size_t(16), 1, None, C.byref(ms), C.byref(units)) == -7
    assert lib.moc_probe(1, fake, C.c_size_t(4096), 1, None, C.byref(ms), C.byref(units)) == -7


def test_outer_route_and_gather_reject_bad_arguments_on_the_host():
    """Every check below fails before the first GPU call, so it runs without a GPU."""
    lib = mb.lib()
    nbytes = C.c_size_t()
    assert lib.moc_outer_workspace_bytes(100, 16, 4, C.byref(nbytes)) == 0 and nbytes.value > 0
    assert lib.moc_outer_workspace_bytes(100, 12, 4, C.byref(nbytes)) == -2        # D not a multiple of 8
    assert lib.moc_outer_workspace_bytes(100, 16, 0, C.byref(nbytes)) == -2        # no segment
    assert lib.moc_outer_workspace_bytes(100, 16, 5000, C.byref(nbytes)) == -2     # more segments than rows
    assert lib.moc_outer_workspace_bytes(100, 16, 4, None) == -1
    fake = C.c_void_p(0x1000)                     # never dereferenced
    off = np.array([0, 10, 40, 100], np.int32)
    sel = np.zeros(3, np.int32); kept = np.zeros(3, np.int32); nk = C.c_int32()

    def call(off_, g=1, M=1, x=fake, dtype=0, D=16, ws_bytes=1 << 30):
        return lib.moc_outer_route(100, D, dtype, x, 3, off_.ctypes.data, None, g, M, 1, fake, fake, sel.ctypes.data,
                                   kept.ctypes.data, C.byref(nk), fake, ws_bytes, None)

    assert call(off, g=3) == -2 and call(off, g=-1) == -2                           # g names no segment
    assert call(off, M=4) == -2 and call(off, M=-1) == -2
    assert call(np.array([0, 10, 10, 100], np.int32)) == -3                         # empty segment
    assert call(np.array([0, 10, 40, 99], np.int32)) == -3                          # does not end at N
    assert call(off, dtype=7) == -6
    assert call(off, x=None) == -1
    assert call(off, x=C.c_void_p(0x1004)) == -8
    assert call(off, ws_bytes=16) == -7

    rg = np.array([[0, 5], [90, 20]], np.int32)                                     # second range runs past the source
    assert lib.moc_gather_rows(1, 100, 64, fake, 2, rg.ctypes.data, fake, fake, 64, None) == -3
    ok = np.array([[0, 5], [90, 10]], np.int32)
    assert lib.moc_gather_rows(1, 100, 60, fake, 2, ok.ctypes.data, fake, fake, 64, None) == -2   # row bytes % 16
    assert lib.moc_gather_rows(1, 100, 64, fake, 2, ok.ctypes.data, fake, fake, 16, None) == -7   # table does not fit
    assert lib.moc_gather_rows(1, 100, 64, None, 2, ok.ctypes.data, fake, fake, 64, None) == -1
    assert lib.moc_gather_rows(1, 100, 64, fake, 0, None, fake, fake, 0, None) == 0               # nothing to do
    empty = np.array([[7, 0], [100, 0]], np.int32)                                  # empty ranges only: nothing to do either
    assert lib.moc_gather_rows(1, 100, 64, None, 2, empty.ctypes.data, None, None, 0, None) == 0
    neg = np.array([[7, -1]], np.int32)
    assert lib.moc_gather_rows(1, 100, 64, fake, 1, neg.ctypes.data, fake, fake, 64, None) == -3
