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
    assert lib.moc_probe(7, fake, C.c_size_t(64), 1, None, C.byref(ms), C.byref(units)) == -2
    assert lib.moc_probe(0, fake, C.c_size_t(64), 0, None, C.byref(ms), C.byref(units)) == -2
    assert lib.moc_probe(0, C.c_void_p(0x1004), C.c_size_t(64), 1, None, C.byref(ms), C.byref(units)) == -8
    assert lib.moc_probe(0, fake, C.c_size_t(16), 1, None, C.byref(ms), C.byref(units)) == -7
    assert lib.moc_probe(1, fake, C.c_size_t(4096), 1, None, C.byref(ms), C.byref(units)) == -7
