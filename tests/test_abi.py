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
    # dominated by [T, 2F] + [T, F] bf16, plus the compacted copies of G, U (loss-mask mode) and the [T, H]-sized rest
    # and the fixed 64 MiB scratch of the split weight-gradient products
    assert 8192 * 3 * 14336 * 2 < n < 3 * 8192 * 3 * 14336 * 2 + (64 << 20)
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


def test_capture_pack_static_rejects_bad_arguments_and_sizes_beyond_its_scratch():
    L = A.lib()
    P = 0x10000
    b = _batch([0, 3, 5])
    st = (B.CStream * 1)(B.CStream(P, P, 8, 8))
    call = lambda **kw: L.alch_capture_pack_static(C.byref(kw.get("b", b)), kw.get("mask", P), kw.get("n", 1), kw.get("st", st),
                                                   kw.get("cap", 5), kw.get("idx", P), kw.get("cu", P), kw.get("status", P), None)
    assert call(mask=None) == -1 and "keep_mask" in _err()
    assert call(idx=None) == -1 and call(cu=None) == -1 and call(status=None) == -1 and call(cap=-1) == -1
    assert call(st=(B.CStream * 1)(B.CStream(P, P, 6, 8))) == -2 and "row_bytes" in _err()
    assert call(b=_batch([0, 3, 2], T=2, max_len=3)) == -2
    # the built-in scratch serves a stated maximum; beyond it the call fails before anything is enqueued
    limit = L.alch_capture_pack_static_max_tokens()
    assert 1 << 24 <= limit < 1 << 31
    assert L.alch_capture_pack_workspace_bytes(limit) <= 64 * 1024 < L.alch_capture_pack_workspace_bytes(limit + 4096)
    assert call(b=_batch([0, limit + 1])) == -5 and "scratch" in _err()


def test_capture_gather_rejects_bad_arguments():
    L = A.lib()
    P = 0x1000
    b = _batch([0, 3, 5])
    st = (B.CStream * 1)(B.CStream(P, P, 16, 16))
    call = lambda **kw: L.alch_capture_gather(C.byref(kw.get("b", b)), kw.get("n", 1), kw.get("st", st), kw.get("cap", 5),
                                              kw.get("idx", P), kw.get("status", P), None)
    assert call(idx=None) == -1 and "kept_index" in _err()
    assert call(status=None) == -1
    assert call(n=-1) == -1 and call(st=None) == -1 and call(cap=-1) == -1
    assert call(st=(B.CStream * 1)(B.CStream(P, P, 6, 16))) == -2
    assert call(st=(B.CStream * 1)(B.CStream(P, None, 16, 16))) == -1
    assert call(b=_batch([0, 3, 2], T=2, max_len=3)) == -2
    assert call(cap=0, idx=None) == 0          # nothing can be written: nothing is launched


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


def test_lora_entry_points_reject_bad_arguments():
    L = A.lib()
    P = 0x10000
    s = A.make_shape(256, 4, 4, 64, 1024, 1e-6, 1e4, "f32")
    b = _batch([0, 128, 256])
    sv, w, g = B.CSaved(*([P] * 9), 0), B.CWeights(*([P] * 9), 0), B.CWgrads(*([None] * 9), 0)

    def lora(rank=8, A_q=P, B_q=P):
        lo = B.CLora(rank=rank, scale=1.0)
        lo.A[0], lo.B[0] = A_q, B_q
        return lo

    def grads(dA_q=None, dA_k=None):
        lg = B.CLoraGrads(accumulate=0)
        lg.dA[0], lg.dA[1] = dA_q, dA_k
        return lg

    call = lambda lo, lg=None, wsb=1 << 40, sv_=sv: L.alch_layer_backward_lora(
        C.byref(s), C.byref(b), C.byref(sv_), C.byref(w), C.byref(lo) if lo is not None else None, P, None, P,
        C.byref(g), C.byref(lg) if lg is not None else None, P, wsb, None)
    assert call(None) == -1 and "lora" in _err()
    assert call(lora(rank=4)) == -2 and "rank" in _err()
    assert call(lora(rank=12)) == -2
    assert call(lora(rank=128)) == -2
    assert call(lora(B_q=None)) == -1 and "both" in _err()
    assert call(lora(A_q=P + 2)) == -1 and "aligned" in _err()
    assert call(lora(), grads(dA_k=P)) == -1 and "without adapter" in _err()   # projection k carries no adapter
    assert call(lora(), grads(dA_q=P), wsb=4096) == -3
    # a record without X2 is fine in general, but not when the output projection is adapted (validated at enqueue
    # time, after the workspace check, so it needs no GPU either: T > 0 and the first launch is never reached)
    q = L.alch_layer_backward_lora_workspace_bytes
    assert q(C.byref(s), 256, 128, 8) > L.alch_layer_backward_workspace_bytes(C.byref(s), 256, 128)
    assert q(C.byref(s), 256, 128, 7) == 0
    assert L.alch_stack_backward_lora_workspace_bytes(C.byref(s), 2, 1000, 256, 128, 8) > q(C.byref(s), 256, 128, 8)

    # stack: the rank must be the same in every layer; the adapter array is required
    sva = (B.CSaved * 2)(sv, sv)
    wa = (B.CWeights * 2)(w, w)
    la = (B.CLora * 2)(lora(rank=8), lora(rank=16))
    sargs = lambda lo: (C.byref(s), 2, 1000, C.byref(b), sva, wa, lo, P, P, P, P, None, None, None, None, None, P, P,
                        None, P, 1 << 40, None)
    assert L.alch_stack_backward_lora(*sargs(la)) == -2 and "rank differs" in _err()
    assert L.alch_stack_backward_lora(*sargs(None)) == -1


def test_shared_prefix_batch_validation():
    L = A.lib()
    P = 0x10000
    s = A.make_shape(256, 4, 4, 64, 1024, 1e-6, 1e4, "f32")
    w, g = B.CWeights(*([P] * 9), 0), B.CWgrads(*([None] * 9), 0)
    sv = B.CSaved(*([P] * 9), 0)
    cu = np.asarray([0, 4, 6, 9], dtype=np.int32)

    def call(prefix, positions=P, dev=P):
        pre = None if prefix is None else np.asarray(prefix, dtype=np.int32)
        b = B.CBatch(3, 9, 4, P, positions, cu.ctypes.data, dev if pre is not None else None,
                     None if pre is None else pre.ctypes.data)
        return L.alch_layer_backward(C.byref(s), C.byref(b), C.byref(sv), C.byref(w), P, None, P, C.byref(g), P, 1024, None)

    assert call([-1, 0, 0]) == -3                      # valid: stops at the workspace check
    assert call([-1, 0, 0], positions=None) == -1 and "positions" in _err()
    assert call([-1, 1, 0]) == -2 and "earlier" in _err()       # a prefix must come before
    assert call([-1, 0, 1]) == -2 and "prefix itself" in _err()  # and have no prefix of its own
    assert call([-2, 0, 0]) == -2
    assert call([-1, 0, 0], dev=None) == -1            # device and host copies go together


def test_forward_from_and_dpo_validation():
    L = A.lib()
    P = 0x10000
    s = A.make_shape(256, 4, 4, 64, 1024, 1e-6, 1e4, "f32")
    w = B.CWeights(*([P] * 9), 0)
    ro = B.CRecordOut(*([P] * 9))
    cu = np.asarray([0, 4, 6, 9], dtype=np.int32)
    pre = np.asarray([-1, 0, 0], dtype=np.int32)
    b = B.CBatch(3, 9, 4, P, P, cu.ctypes.data, P, pre.ctypes.data)
    fwd = lambda batch, seq_begin, ws=1024: L.alch_layer_forward_from(C.byref(s), C.byref(batch), seq_begin, P, C.byref(w), P,
                                                                       C.byref(ro), P, ws, None)
    assert fwd(b, 1) == -3                                   # valid: stops at the workspace check
    assert fwd(b, 3, 1 << 30) == 0                           # no sequence left: nothing is launched
    assert fwd(b, 4) == -1 and "seq_begin" in _err()
    assert fwd(b, -1) == -1
    nopos = B.CBatch(3, 9, 4, P, None, cu.ctypes.data, None, None)
    assert fwd(nopos, 1) == -1 and "positions" in _err()
    assert fwd(nopos, 0) == -3

    sv, g = B.CSaved(*([P] * 9), 0), B.CWgrads(*([None] * 9), 0)
    rows = np.asarray([3, 3, 4, 6], dtype=np.int32)

    def dpo_call(d):
        return L.alch_stack_backward_dpo(C.byref(s), 1, 100, C.byref(b), C.byref(sv), C.byref(w), None, P, P, P,
                                         C.byref(d) if d is not None else None, C.byref(g), None, None, None, P, P, None,
                                         P, 1024, None)
    ok = B.CDpo(4, 1, P, P, P, rows.ctypes.data, P, 0.1, None)
    assert dpo_call(ok) == -3
    assert dpo_call(None) == -1 and "dpo is NULL" in _err()
    assert dpo_call(B.CDpo(4, 1, P, P, P, None, P, 0.1, None)) == -1
    assert dpo_call(B.CDpo(4, 1, P, P, P, rows.ctypes.data, None, 0.1, None)) == -1 and "ref_logp" in _err()
    assert dpo_call(B.CDpo(10, 1, P, P, P, rows.ctypes.data, P, 0.1, None)) == -2      # more items than tokens
    bad = np.asarray([3, 2, 4, 6], dtype=np.int32)
    assert dpo_call(B.CDpo(4, 1, P, P, P, bad.ctypes.data, P, 0.1, None)) == -2 and "ascending" in _err()
    far = np.asarray([3, 3, 4, 9], dtype=np.int32)
    assert dpo_call(B.CDpo(4, 1, P, P, P, far.ctypes.data, P, 0.1, None)) == -2 and "outside" in _err()
    assert dpo_call(B.CDpo(0, 0, None, None, None, None, None, 0.1, None)) == -3       # nothing scored is legal


def test_six_stream_record_passes_validation_but_missing_required_tensors_do_not():
    L = A.lib()
    P = 0x10000
    s = A.make_shape(256, 4, 4, 64, 1024, 1e-6, 1e4, "f32")
    b = _batch([0, 128, 256])
    w, g = B.CWeights(*([P] * 9), 0), B.CWgrads(*([None] * 9), 0)
    # field order X, X2, Q, K, V, O, G, U, LSE: X2, O, LSE may be NULL -> validation passes, the call then stops at
    # the workspace check (-3) before anything is launched
    six = B.CSaved(P, None, P, P, P, None, P, P, None, 0)
    assert L.alch_layer_backward(C.byref(s), C.byref(b), C.byref(six), C.byref(w), P, None, P, C.byref(g), P, 1024, None) == -3
    # layer input, query and KV cache alone: G and U may be NULL too
    four = B.CSaved(P, None, P, P, P, None, None, None, None, 0)
    assert L.alch_layer_backward(C.byref(s), C.byref(b), C.byref(four), C.byref(w), P, None, P, C.byref(g), P, 1024, None) == -3
    for missing in (0, 2, 3, 4):  # X, Q, K, V are required
        ptrs = [P] * 9
        ptrs[missing] = None
        sv = B.CSaved(*ptrs, 0)
        assert L.alch_layer_backward(C.byref(s), C.byref(b), C.byref(sv), C.byref(w), P, None, P, C.byref(g), P, 1 << 40, None) == -1


def test_gemm_rejects_bad_arguments():
    L = A.lib()
    P = 0x10000
    term = (B.CGemmTerm * 1)(B.CGemmTerm(P, P, 64, 64, 256))
    call = lambda **kw: L.alch_gemm_ws(kw.get("dtype", 1), kw.get("M", 256), kw.get("N", 256), 1, 0, kw.get("n_terms", 1),
                                       kw.get("terms", term), kw.get("C", P), kw.get("ldc", 256), 0, kw.get("ws", None),
                                       kw.get("ws_bytes", 0), None)
    assert L.alch_gemm_workspace_bytes() == 64 << 20
    assert call(dtype=7) == -1
    assert call(M=-1) == -2
    assert call(n_terms=0) == -1 and call(n_terms=5) == -1 and call(terms=None) == -1
    assert call(C=None) == -1 and call(ldc=8) == -1
    assert call(ws=P + 4, ws_bytes=64 << 20) == -1 and "workspace" in _err()
    bad = (B.CGemmTerm * 1)(B.CGemmTerm(P, P, 64, 32, 256))      # lda < K of a k-major operand
    assert call(terms=bad) == -2
    assert call(M=0) == 0                                           # nothing to do, nothing launched


def test_header_is_plain_c_and_links_from_c(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 on its own, and a C program must link against the
    # library and reach an entry point that needs no GPU
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    hdr = os.path.join(root, "include", "alch.h")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", hdr], check=True)
    src = tmp_path / "t.c"
    src.write_text(r"""
#include "alch.h"
#include <stdio.h>
int main(void) {
    printf("%s %lu\n", alch_version(), (unsigned long)alch_gemm_workspace_bytes());
    return alch_gemm(ALCH_BF16, -1, 4, 1, 0, 1, 0, 0, 4, 0, 0) == ALCH_ERR_SHAPE ? 0 : 1;
}
""")
    exe = tmp_path / "t"
    lib = A.library_path()
    subprocess.run([gcc, "-std=c99", "-I", os.path.join(root, "include"), str(src), "-o", str(exe), lib,
                    "-Wl,-rpath," + os.path.dirname(lib)], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.startswith("alch ")
