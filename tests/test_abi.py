"""CPU-only checks of the C ABI: the library loads, exports every symbol include/alch.h
declares, and rejects bad arguments on the host before any GPU work."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2503_01066_amd as A
from paper_2503_01066_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "alch.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(alch_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = A.lib()
    names = declared_symbols()
    assert {"alch_capture_pack", "alch_layer_backward", "alch_stack_backward", "alch_last_error"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
    assert b"gfx950" in L.alch_version()


def _batch(cu, T=None, max_len=None):
    cu = np.asarray(cu, dtype=np.int32)
    b = B.CBatch(len(cu) - 1, int(cu[-1]) if T is None else T,
                 int(np.diff(cu).max()) if max_len is None else max_len, 0x1000, 0, cu.ctypes.data)
    b._keep = cu
    return b


def _err():
    return A.lib().alch_last_error().decode()


def test_workspace_queries():
    L = A.lib()
    s = A.make_shape(4096, 32, 8, 128, 14336, 1e-5, 5e5, "bf16")
    n = L.alch_layer_backward_workspace_bytes(C.byref(s), 8192, 2048)
    # dominated by [T, 2F] + [T, F] bf16
    assert 8192 * 3 * 14336 * 2 < n < 2 * 8192 * 3 * 14336 * 2
    assert L.alch_layer_backward_workspace_bytes(C.byref(s), 0, 0) > 0
    bad = A.make_shape(4096, 32, 7, 128, 14336, 1e-5, 5e5, "bf16")
    assert L.alch_layer_backward_workspace_bytes(C.byref(bad), 8192, 2048) == 0
    assert L.alch_capture_pack_workspace_bytes(0) >= 256
    assert L.alch_capture_pack_workspace_bytes(1 << 20) >= (1 << 20) // 4096 * 4
    assert L.alch_stack_backward_workspace_bytes(C.byref(s), 32, 128256, 1024, 512) > n // 16


def test_capture_pack_rejects_bad_arguments():
    L = A.lib()
    P = 0x10000  # fake, aligned, never dereferenced: validation fails first
    b = _batch([0, 3, 5])
    st = (B.CStream * 1)(B.CStream(P, P, 6, 8))
    assert L.alch_capture_pack(C.byref(b), P, 1, st, 5, P, P, P, P, 1024, None) == -2 and "row_bytes" in _err()
    st = (B.CStream * 1)(B.CStream(P, P, 8, 4))
    assert L.alch_capture_pack(C.byref(b), P, 1, st, 5, P, P, P, P, 1024, None) == -2
    st = (B.CStream * 1)(B.CStream(P, P, 8, 8))
    assert L.alch_capture_pack(C.byref(b), None, 1, st, 5, P, P, P, P, 1024, None) == -1 and "keep_mask" in _err()
    assert L.alch_capture_pack(C.byref(b), P, 1, st, 5, P, P, P, None, 0, None) == -3
    assert L.alch_capture_pack(C.byref(b), P, 1, st, -1, P, P, P, P, 1024, None) == -1
    assert L.alch_capture_pack(C.byref(_batch([0, 3, 2], T=2, max_len=3)), P, 1, st, 5, P, P, P, P, 1024, None) == -2
    assert L.alch_capture_pack(C.byref(_batch([0, 3, 5], T=6)), P, 1, st, 5, P, P, P, P, 1024, None) == -2
    assert L.alch_capture_pack(C.byref(_batch([1, 3, 5])), P, 1, st, 5, P, P, P, P, 1024, None) == -2
    assert L.alch_capture_pack(None, P, 1, st, 5, P, P, P, P, 1024, None) == -1


def test_layer_backward_rejects_bad_arguments():
    L = A.lib()
    P = 0x10000
    s = A.make_shape(256, 4, 4, 64, 1024, 1e-6, 1e4, "f32")
    b = _batch([0, 128, 256])
    sv = B.CSaved(*([P] * 9), 7)
    w = B.CWeights(*([P] * 9), 7)
    g = B.CWgrads(*([P] * 9), 0)
    big = 1 << 40
    call = lambda **kw: L.alch_layer_backward(C.byref(kw.get("s", s)), C.byref(kw.get("b", b)),
                                              C.byref(kw.get("sv", sv)), C.byref(kw.get("w", w)), kw.get("dY", P),
                                              None, kw.get("dX", P), C.byref(g), kw.get("ws", P),
                                              kw.get("wsb", big), None)
    assert call(w=B.CWeights(*([P] * 9), 8)) == -4 and "version" in _err()          # stale record
    assert call(s=A.make_shape(256, 4, 3, 64, 1024, 1e-6, 1e4, "f32")) == -2
    assert call(s=A.make_shape(256, 4, 4, 63, 1024, 1e-6, 1e4, "f32")) == -2
    assert call(s=A.make_shape(256, 4, 4, 512, 1024, 1e-6, 1e4, "f32")) == -5
    assert call(s=B.LayerShape(256, 4, 4, 64, 1024, 1e-6, 1e4, 9)) == -1
    assert call(dY=None) == -1 and "dY" in _err()
    assert call(dX=P + 4) == -1 and "aligned" in _err()
    assert call(wsb=1024) == -3
    assert call(ws=None) == -3
    assert call(sv=B.CSaved(P, P, P, None, P, P, P, P, P, 7)) == -1 and "saved.K" in _err()
    assert call(b=_batch([0, 128, 256], max_len=100)) == -2 and "max_seqlen" in _err()


def test_stack_backward_rejects_bad_arguments():
    L = A.lib()
    P = 0x10000
    s = A.make_shape(256, 4, 4, 64, 1024, 1e-6, 1e4, "f32")
    b = _batch([0, 128, 256])
    sv = (B.CSaved * 2)(B.CSaved(*([P] * 9), 0), B.CSaved(*([P] * 9), 1))
    w = (B.CWeights * 2)(B.CWeights(*([P] * 9), 0), B.CWeights(*([P] * 9), 0))
    args = lambda **kw: (C.byref(s), 2, kw.get("vocab", 1000), C.byref(b), sv, w, P, P, P, kw.get("labels", P), None,
                         None, None, None, P, kw.get("loss", P), None, P, kw.get("wsb", 1 << 40), None)
    assert L.alch_stack_backward(*args()) == -4          # layer 1 record is stale
    sv[1].weights_version = 0
    assert L.alch_stack_backward(*args(vocab=0)) == -2
    assert L.alch_stack_backward(*args(labels=None)) == -1
    assert L.alch_stack_backward(*args(wsb=4096)) == -3


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_LIB", None)
    monkeypatch.setattr(B, "library_path", lambda: "/nonexistent/libalch.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        B.lib()
