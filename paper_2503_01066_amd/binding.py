"""ctypes binding of libalch.so: argument marshalling only.

Tensors are torch tensors on the GPU (torch is used for device memory and streams);
every step of the computation runs inside the library.  There is no fallback: if the
library has not been built, loading raises.
"""
import ctypes as C
import os

import numpy as np
import torch

RECORD_KEYS = ("X", "X2", "Q", "K", "V", "O", "G", "U")  # + LSE (fp32)
WEIGHT_KEYS = ("Wq", "Wk", "Wv", "Wo", "Wg", "Wu", "Wd", "g1", "g2")
STATUS = {0: "ALCH_OK", -1: "ALCH_ERR_INVALID_ARG", -2: "ALCH_ERR_SHAPE", -3: "ALCH_ERR_WORKSPACE",
          -4: "ALCH_ERR_STALE", -5: "ALCH_ERR_UNSUPPORTED", -6: "ALCH_ERR_HIP", -7: "ALCH_ERR_ABORTED"}
ALCH_F32, ALCH_BF16 = 0, 1


class AlchError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("%s: %s" % (STATUS.get(code, code), message))
        self.code = code
        self.message = message


class LayerShape(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("rms_eps", C.c_float),
                ("rope_base", C.c_float), ("dtype", C.c_int)]


class CBatch(C.Structure):
    _fields_ = [("n_seqs", C.c_int32), ("total_tokens", C.c_int32), ("max_seqlen", C.c_int32),
                ("cu_seqlens", C.c_void_p), ("positions", C.c_void_p), ("cu_seqlens_host", C.c_void_p),
                ("seq_prefix", C.c_void_p), ("seq_prefix_host", C.c_void_p)]


class CStream(C.Structure):
    _fields_ = [("src", C.c_void_p), ("dst", C.c_void_p), ("row_bytes", C.c_size_t),
                ("src_row_stride_bytes", C.c_size_t)]


class CSaved(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in RECORD_KEYS] + [("LSE", C.c_void_p), ("weights_version", C.c_uint64)]


class CWeights(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in WEIGHT_KEYS] + [("weights_version", C.c_uint64)]


class CWgrads(C.Structure):
    _fields_ = [("d" + k, C.c_void_p) for k in WEIGHT_KEYS] + [("accumulate", C.c_int32)]


PROJECTIONS = ("q", "k", "v", "o", "g", "u", "d")  # order of the adapter arrays


class CLora(C.Structure):
    _fields_ = [("rank", C.c_int32), ("scale", C.c_float), ("A", C.c_void_p * 7), ("B", C.c_void_p * 7)]


class CLoraGrads(C.Structure):
    _fields_ = [("dA", C.c_void_p * 7), ("dB", C.c_void_p * 7), ("accumulate", C.c_int32)]


class CRecordOut(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in RECORD_KEYS] + [("LSE", C.c_void_p)]


class CGemmTerm(C.Structure):
    _fields_ = [("A", C.c_void_p), ("B", C.c_void_p), ("K", C.c_int32), ("lda", C.c_int64), ("ldb", C.c_int64)]


class CTraceRecord(C.Structure):
    _fields_ = [("kind", C.c_int32), ("flops", C.c_double), ("bytes", C.c_double), ("ms", C.c_float)]


TRACE_KINDS = ("gemm_mfma", "gemm_generic", "pack_scan", "pack_gather", "attn_bwd", "attn_fwd", "row_ops",
               "cross_entropy", "lora")

HOOK_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_int)


class CHooks(C.Structure):
    _fields_ = [("layer_ready", HOOK_FN), ("preempt", HOOK_FN), ("user", C.c_void_p)]


def library_path():
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libalch.so")


_LIB = None


def lib():
    """Loads libalch.so (built by paper_2503_01066_amd.build); raises if it is missing."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError("libalch.so not found at %s: run `python -m paper_2503_01066_amd.build` "
                           "(there is no fallback path)" % path)
    L = C.CDLL(path)
    L.alch_last_error.restype = C.c_char_p
    L.alch_version.restype = C.c_char_p
    for name in ("alch_capture_pack_workspace_bytes", "alch_layer_backward_workspace_bytes",
                 "alch_stack_backward_workspace_bytes", "alch_layer_forward_workspace_bytes"):
        getattr(L, name).restype = C.c_size_t
    L.alch_capture_pack_workspace_bytes.argtypes = [C.c_int32]
    L.alch_layer_backward_workspace_bytes.argtypes = [C.POINTER(LayerShape), C.c_int32, C.c_int32]
    L.alch_layer_forward_workspace_bytes.argtypes = [C.POINTER(LayerShape), C.c_int32, C.c_int32]
    L.alch_stack_backward_workspace_bytes.argtypes = [C.POINTER(LayerShape), C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    L.alch_capture_pack.restype = C.c_int
    L.alch_capture_pack.argtypes = [C.POINTER(CBatch), C.c_void_p, C.c_int32, C.POINTER(CStream), C.c_int64,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.alch_capture_pack_static.restype = C.c_int
    L.alch_capture_pack_static.argtypes = [C.POINTER(CBatch), C.c_void_p, C.c_int32, C.POINTER(CStream), C.c_int64,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.alch_capture_pack_static_max_tokens.restype = C.c_size_t
    L.alch_capture_pack_static_max_tokens.argtypes = []
    L.alch_capture_gather.restype = C.c_int
    L.alch_capture_gather.argtypes = [C.POINTER(CBatch), C.c_int32, C.POINTER(CStream), C.c_int64, C.c_void_p,
                                      C.c_void_p, C.c_void_p]
    L.alch_layer_backward.restype = C.c_int
    L.alch_layer_backward.argtypes = [C.POINTER(LayerShape), C.POINTER(CBatch), C.POINTER(CSaved),
                                      C.POINTER(CWeights), C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.POINTER(CWgrads), C.c_void_p, C.c_size_t, C.c_void_p]
    L.alch_layer_backward_lora_workspace_bytes.restype = C.c_size_t
    L.alch_layer_backward_lora_workspace_bytes.argtypes = [C.POINTER(LayerShape), C.c_int32, C.c_int32, C.c_int32]
    L.alch_layer_backward_lora.restype = C.c_int
    L.alch_layer_backward_lora.argtypes = [C.POINTER(LayerShape), C.POINTER(CBatch), C.POINTER(CSaved),
                                           C.POINTER(CWeights), C.POINTER(CLora), C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.POINTER(CWgrads), C.POINTER(CLoraGrads), C.c_void_p, C.c_size_t, C.c_void_p]
    L.alch_stack_backward.restype = C.c_int
    L.alch_stack_backward.argtypes = [C.POINTER(LayerShape), C.c_int32, C.c_int32, C.POINTER(CBatch),
                                      C.POINTER(CSaved), C.POINTER(CWeights), C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.POINTER(CWgrads), C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.POINTER(CHooks), C.c_void_p, C.c_size_t, C.c_void_p]
    L.alch_stack_backward_lora_workspace_bytes.restype = C.c_size_t
    L.alch_stack_backward_lora_workspace_bytes.argtypes = [C.POINTER(LayerShape), C.c_int32, C.c_int32, C.c_int32,
                                                           C.c_int32, C.c_int32]
    L.alch_stack_backward_lora.restype = C.c_int
    L.alch_stack_backward_lora.argtypes = [C.POINTER(LayerShape), C.c_int32, C.c_int32, C.POINTER(CBatch),
                                           C.POINTER(CSaved), C.POINTER(CWeights), C.POINTER(CLora), C.c_void_p,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(CWgrads),
                                           C.POINTER(CLoraGrads), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.POINTER(CHooks), C.c_void_p, C.c_size_t, C.c_void_p]
    L.alch_layer_forward.restype = C.c_int
    L.alch_layer_forward.argtypes = [C.POINTER(LayerShape), C.POINTER(CBatch), C.c_void_p, C.POINTER(CWeights),
                                     C.c_void_p, C.POINTER(CRecordOut), C.c_void_p, C.c_size_t, C.c_void_p]
    L.alch_stack_backward_dpo.restype = C.c_int
    L.alch_stack_backward_dpo.argtypes = [C.POINTER(LayerShape), C.c_int32, C.c_int32, C.POINTER(CBatch),
                                          C.POINTER(CSaved), C.POINTER(CWeights), C.POINTER(CLora), C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.POINTER(CDpo), C.POINTER(CWgrads),
                                          C.POINTER(CLoraGrads), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.POINTER(CHooks), C.c_void_p, C.c_size_t, C.c_void_p]
    L.alch_layer_forward_from.restype = C.c_int
    L.alch_layer_forward_from.argtypes = [C.POINTER(LayerShape), C.POINTER(CBatch), C.c_int32, C.c_void_p,
                                          C.POINTER(CWeights), C.c_void_p, C.POINTER(CRecordOut), C.c_void_p,
                                          C.c_size_t, C.c_void_p]
    L.alch_gemm.restype = C.c_int
    L.alch_gemm.argtypes = [C.c_int, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(CGemmTerm),
                            C.c_void_p, C.c_int64, C.c_int32, C.c_void_p]
    L.alch_gemm_ws.restype = C.c_int
    L.alch_gemm_ws.argtypes = [C.c_int, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(CGemmTerm),
                               C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
    L.alch_gemm_workspace_bytes.restype = C.c_size_t
    L.alch_gemm_workspace_bytes.argtypes = []
    L.alch_attention_forward.restype = C.c_int
    L.alch_attention_forward.argtypes = [C.POINTER(LayerShape), C.POINTER(CBatch), C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_void_p]
    L.alch_trace_enable.argtypes = [C.c_int32]
    L.alch_trace_collect.argtypes = [C.POINTER(CTraceRecord), C.c_int32, C.POINTER(C.c_int32)]
    _LIB = L
    return L


def _check(rc):
    if rc != 0:
        raise AlchError(rc, lib().alch_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_handle(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def make_shape(hidden, n_q_heads, n_kv_heads, head_dim, ffn, rms_eps, rope_base, dtype):
    code = {"bf16": ALCH_BF16, "f32": ALCH_F32, torch.bfloat16: ALCH_BF16, torch.float32: ALCH_F32}[dtype]
    return LayerShape(hidden, n_q_heads, n_kv_heads, head_dim, ffn, rms_eps, rope_base, code)


def _torch_dtype(shape):
    return torch.bfloat16 if shape.dtype == ALCH_BF16 else torch.float32


class Batch:
    """A ragged batch: host cu_seqlens (int32 numpy) mirrored on the device.  prefix: per sequence -1 or the
    index of the earlier sequence whose tokens it also attends to (positions must then be given)."""

    def __init__(self, cu_seqlens, device="cuda", positions=None, prefix=None):
        self.cu_host = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
        self.n_seqs = int(self.cu_host.shape[0] - 1)
        self.total_tokens = int(self.cu_host[-1])
        lens = np.diff(self.cu_host)
        self.max_seqlen = int(lens.max()) if self.n_seqs > 0 else 0
        self.cu_dev = torch.from_numpy(self.cu_host.copy()).to(device)
        self.positions = None if positions is None else torch.as_tensor(positions, dtype=torch.int32).to(device)
        self.prefix_host = None if prefix is None else np.ascontiguousarray(prefix, dtype=np.int32)
        self.prefix_dev = None if prefix is None else torch.from_numpy(self.prefix_host.copy()).to(device)
        self.c = CBatch(self.n_seqs, self.total_tokens, self.max_seqlen, self.cu_dev.data_ptr(),
                        0 if self.positions is None else self.positions.data_ptr(), self.cu_host.ctypes.data,
                        None if prefix is None else self.prefix_dev.data_ptr(),
                        None if prefix is None else self.prefix_host.ctypes.data)


def _workspace(nbytes, device):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def alch_capture_pack(batch, keep_mask, streams, capacity=None, dsts=None, stream=None, workspace=None):
    """streams: list of 2-D device tensors [T, width] (row-contiguous; the row stride may exceed the
    width, e.g. a column slice of a fused buffer).  Returns (kept_index, cu_kept, n_kept_and_status, dsts)."""
    L = lib()
    T = batch.total_tokens
    dev = keep_mask.device
    capacity = T if capacity is None else int(capacity)
    if dsts is None:
        dsts = [torch.empty((capacity, s.shape[1]), dtype=s.dtype, device=dev) for s in streams]
    arr = (CStream * max(len(streams), 1))()
    for i, (s, d) in enumerate(zip(streams, dsts)):
        assert s.numel() == 0 or (s.stride(1) == 1 and d.is_contiguous())
        row_stride = s.stride(0) if s.numel() > 0 else s.shape[1]
        arr[i] = CStream(s.data_ptr(), d.data_ptr(), s.shape[1] * s.element_size(), row_stride * s.element_size())
    kept_index = torch.empty(max(capacity, 1), dtype=torch.int32, device=dev)
    cu_kept = torch.empty(batch.n_seqs + 1, dtype=torch.int32, device=dev)
    status = torch.empty(2, dtype=torch.int32, device=dev)
    need = L.alch_capture_pack_workspace_bytes(T)
    ws = workspace if workspace is not None else _workspace(need, dev)
    _check(L.alch_capture_pack(C.byref(batch.c), _ptr(keep_mask), len(streams), arr, capacity, _ptr(kept_index),
                               _ptr(cu_kept), _ptr(status), _ptr(ws), ws.numel(), _stream_handle(stream)))
    return kept_index, cu_kept, status, dsts


def alch_capture_pack_static(batch, keep_mask, streams, dsts, kept_index, cu_kept, status, stream=None):
    """alch_capture_pack on the library's built-in scratch: every buffer, outputs included, comes from the
    caller, and neither this wrapper nor the library allocates device memory."""
    L = lib()
    arr = (CStream * max(len(streams), 1))()
    for i, (s, d) in enumerate(zip(streams, dsts)):
        assert s.numel() == 0 or (s.stride(1) == 1 and d.is_contiguous())
        row_stride = s.stride(0) if s.numel() > 0 else s.shape[1]
        arr[i] = CStream(s.data_ptr(), d.data_ptr(), s.shape[1] * s.element_size(), row_stride * s.element_size())
    capacity = min([int(kept_index.numel())] + [int(d.shape[0]) for d in dsts])
    _check(L.alch_capture_pack_static(C.byref(batch.c), _ptr(keep_mask), len(streams), arr, capacity,
                                      _ptr(kept_index), _ptr(cu_kept), _ptr(status), _stream_handle(stream)))
    return capacity


def alch_capture_gather(batch, kept_index, status, streams, capacity=None, dsts=None, stream=None):
    """Gathers further streams with the index of an earlier alch_capture_pack on the same batch and mask
    (kept_index, status = its second and third return values).  Returns dsts."""
    L = lib()
    dev = kept_index.device
    capacity = batch.total_tokens if capacity is None else int(capacity)
    if dsts is None:
        dsts = [torch.empty((capacity, s.shape[1]), dtype=s.dtype, device=dev) for s in streams]
    arr = (CStream * max(len(streams), 1))()
    for i, (s, d) in enumerate(zip(streams, dsts)):
        assert s.numel() == 0 or (s.stride(1) == 1 and d.is_contiguous())
        row_stride = s.stride(0) if s.numel() > 0 else s.shape[1]
        arr[i] = CStream(s.data_ptr(), d.data_ptr(), s.shape[1] * s.element_size(), row_stride * s.element_size())
    _check(L.alch_capture_gather(C.byref(batch.c), len(streams), arr, capacity, _ptr(kept_index), _ptr(status),
                                 _stream_handle(stream)))
    return dsts


def _saved_struct(saved, version):
    # X2, O and LSE may be absent (six-stream record): the library recomputes them
    ptr = lambda k: saved[k].data_ptr() if saved.get(k) is not None else None
    return CSaved(*[ptr(k) for k in RECORD_KEYS], ptr("LSE"), version)


def _weights_struct(weights, version):
    return CWeights(*[weights[k].data_ptr() for k in WEIGHT_KEYS], version)


def _wgrads_struct(grads, accumulate):
    return CWgrads(*[(grads[k].data_ptr() if grads.get(k) is not None else None) for k in
                     ("d" + w for w in WEIGHT_KEYS)], 1 if accumulate else 0)


def layer_backward_workspace_bytes(shape, total_tokens, max_seqlen):
    return lib().alch_layer_backward_workspace_bytes(C.byref(shape), total_tokens, max_seqlen)


def stack_backward_workspace_bytes(shape, n_layers, vocab, total_tokens, max_seqlen):
    return lib().alch_stack_backward_workspace_bytes(C.byref(shape), n_layers, vocab, total_tokens, max_seqlen)


def alch_layer_backward(shape, batch, saved, weights, dY, loss_mask=None, want=WEIGHT_KEYS, grads=None,
                        accumulate=False, dX=None, workspace=None, stream=None, saved_version=0, weights_version=0):
    """Returns dict with dX and the requested weight gradients ('dWq', ...)."""
    L = lib()
    dev = dY.device
    if grads is None:
        grads = {"d" + k: torch.empty_like(weights[k]) for k in want}
    if dX is None:
        dX = torch.empty_like(dY)
    need = L.alch_layer_backward_workspace_bytes(C.byref(shape), batch.total_tokens, batch.max_seqlen)
    ws = workspace if workspace is not None else _workspace(need, dev)
    sv, w, g = _saved_struct(saved, saved_version), _weights_struct(weights, weights_version), _wgrads_struct(grads, accumulate)
    _check(L.alch_layer_backward(C.byref(shape), C.byref(batch.c), C.byref(sv), C.byref(w), _ptr(dY), _ptr(loss_mask),
                                 _ptr(dX), C.byref(g), _ptr(ws), ws.numel(), _stream_handle(stream)))
    out = dict(grads)
    out["dX"] = dX
    return out


def alch_layer_backward_lora(shape, batch, saved, weights, lora, rank, scale, dY, loss_mask=None, want=(), grads=None,
                             lora_grads=None, accumulate=False, dX=None, workspace=None, stream=None):
    """Layer backward with low-rank adapters.  lora: dict projection -> (A [rank, in], B [out, rank]) for the
    adapted projections among PROJECTIONS.  want: base weight gradients to produce (default none: frozen base).
    lora_grads: dict 'dAq', 'dBq', ... -> tensor (default: all adapters).  Returns dict with dX, the base
    gradients asked for and the adapter gradients."""
    L = lib()
    dev = dY.device
    if grads is None:
        grads = {"d" + k: torch.empty_like(weights[k]) for k in want}
    if lora_grads is None:
        lora_grads = {}
        for p_, (A_, B_) in lora.items():
            lora_grads["dA" + p_] = torch.empty_like(A_)
            lora_grads["dB" + p_] = torch.empty_like(B_)
    if dX is None:
        dX = torch.empty_like(dY)
    cl, cg = _lora_structs(lora, lora_grads, rank, scale, accumulate)
    need = L.alch_layer_backward_lora_workspace_bytes(C.byref(shape), batch.total_tokens, batch.max_seqlen, rank)
    ws = workspace if workspace is not None else _workspace(need, dev)
    sv, w, g = _saved_struct(saved, 0), _weights_struct(weights, 0), _wgrads_struct(grads, accumulate)
    _check(L.alch_layer_backward_lora(C.byref(shape), C.byref(batch.c), C.byref(sv), C.byref(w), C.byref(cl), _ptr(dY),
                                      _ptr(loss_mask), _ptr(dX), C.byref(g), C.byref(cg), _ptr(ws), ws.numel(),
                                      _stream_handle(stream)))
    out = dict(grads)
    out.update(lora_grads)
    out["dX"] = dX
    return out


def alch_layer_forward(shape, batch, X, weights, workspace=None, stream=None, seq_begin=0, rec=None, Y=None):
    """Runs the layer forward; returns (Y, record dict incl. LSE).  seq_begin > 0: only the sequences from
    seq_begin on are computed (alch_layer_forward_from); rec and Y then hold the earlier rows already."""
    L = lib()
    dev, dt = X.device, X.dtype
    T = batch.total_tokens
    QD, KD = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    widths = dict(X=shape.hidden, X2=shape.hidden, Q=QD, K=KD, V=KD, O=QD, G=shape.ffn, U=shape.ffn)
    if rec is None:
        rec = {k: torch.empty((T, w), dtype=dt, device=dev) for k, w in widths.items()}
        rec["LSE"] = torch.empty((T, shape.n_q_heads), dtype=torch.float32, device=dev)
    if Y is None:
        Y = torch.empty_like(X)
    need = L.alch_layer_forward_workspace_bytes(C.byref(shape), T, batch.max_seqlen)
    ws = workspace if workspace is not None else _workspace(need, dev)
    ro = CRecordOut(*[rec[k].data_ptr() for k in RECORD_KEYS], rec["LSE"].data_ptr())
    w = _weights_struct(weights, 0)
    if seq_begin:
        _check(L.alch_layer_forward_from(C.byref(shape), C.byref(batch.c), seq_begin, _ptr(X), C.byref(w), _ptr(Y),
                                         C.byref(ro), _ptr(ws), ws.numel(), _stream_handle(stream)))
    else:
        _check(L.alch_layer_forward(C.byref(shape), C.byref(batch.c), _ptr(X), C.byref(w), _ptr(Y), C.byref(ro),
                                    _ptr(ws), ws.numel(), _stream_handle(stream)))
    return Y, rec


def alch_stack_backward(shape, batch, saved_layers, weights_layers, X_final, g_final, W_lm, labels, loss_mask=None,
                        want=WEIGHT_KEYS, grads_layers=None, accumulate=False, want_head=True, hooks=None,
                        workspace=None, stream=None):
    """Returns dict: loss (device float tensor [1]), dX_embed, dg_final, dW_lm, layers=[grad dicts]."""
    L = lib()
    dev = X_final.device
    n_layers = len(saved_layers)
    vocab = W_lm.shape[0]
    if grads_layers is None:
        grads_layers = [{"d" + k: torch.empty_like(w[k]) for k in want} for w in weights_layers]
    SA = (CSaved * max(n_layers, 1))(*[_saved_struct(s, 0) for s in saved_layers])
    WA = (CWeights * max(n_layers, 1))(*[_weights_struct(w, 0) for w in weights_layers])
    GA = (CWgrads * max(n_layers, 1))(*[_wgrads_struct(g, accumulate) for g in grads_layers])
    dg_final = torch.empty_like(g_final) if want_head else None
    dW_lm = torch.empty_like(W_lm) if want_head else None
    dX_embed = torch.empty_like(X_final)
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    need = L.alch_stack_backward_workspace_bytes(C.byref(shape), n_layers, vocab, batch.total_tokens, batch.max_seqlen)
    ws = workspace if workspace is not None else _workspace(need, dev)
    hk = None
    if hooks is not None:
        ready, preempt = hooks
        hk = CHooks(HOOK_FN(ready) if ready else HOOK_FN(), HOOK_FN(preempt) if preempt else HOOK_FN(), None)
    _check(L.alch_stack_backward(C.byref(shape), n_layers, vocab, C.byref(batch.c), SA, WA, _ptr(X_final),
                                 _ptr(g_final), _ptr(W_lm), _ptr(labels), _ptr(loss_mask), GA, _ptr(dg_final),
                                 _ptr(dW_lm), _ptr(dX_embed), _ptr(loss), C.byref(hk) if hk else None, _ptr(ws),
                                 ws.numel(), _stream_handle(stream)))
    return dict(loss=loss, dX_embed=dX_embed, dg_final=dg_final, dW_lm=dW_lm, layers=grads_layers)


def _lora_structs(lora, lora_grads, rank, scale, accumulate):
    cl = CLora(rank=rank, scale=scale)
    cg = CLoraGrads(accumulate=1 if accumulate else 0)
    for i, p_ in enumerate(PROJECTIONS):
        if p_ in lora:
            cl.A[i], cl.B[i] = lora[p_][0].data_ptr(), lora[p_][1].data_ptr()
        for arr, key in ((cg.dA, "dA" + p_), (cg.dB, "dB" + p_)):
            if lora_grads.get(key) is not None:
                arr[i] = lora_grads[key].data_ptr()
    return cl, cg


def alch_stack_backward_lora(shape, batch, saved_layers, weights_layers, lora_layers, rank, scale, X_final, g_final,
                             W_lm, labels, loss_mask=None, want=(), want_head=False, lora_grads_layers=None,
                             grads_layers=None, accumulate=False, hooks=None, workspace=None, stream=None):
    """Stack backward with adapters.  lora_layers: list of dicts projection -> (A, B).  Defaults: frozen base and
    frozen head (want=(), want_head=False), gradients of every adapter.  Returns the dict of alch_stack_backward;
    the per-layer dicts hold the adapter gradients ('dAq', 'dBq', ...) and any base gradients asked for."""
    L = lib()
    dev = X_final.device
    n_layers = len(saved_layers)
    vocab = W_lm.shape[0]
    if grads_layers is None:
        grads_layers = [{"d" + k: torch.empty_like(w[k]) for k in want} for w in weights_layers]
    if lora_grads_layers is None:
        lora_grads_layers = []
        for lo in lora_layers:
            g = {}
            for p_, (A_, B_) in lo.items():
                g["dA" + p_], g["dB" + p_] = torch.empty_like(A_), torch.empty_like(B_)
            lora_grads_layers.append(g)
    n = max(n_layers, 1)
    SA = (CSaved * n)(*[_saved_struct(s, 0) for s in saved_layers])
    WA = (CWeights * n)(*[_weights_struct(w, 0) for w in weights_layers])
    GA = (CWgrads * n)(*[_wgrads_struct(g, accumulate) for g in grads_layers])
    pairs = [_lora_structs(lo, lg, rank, scale, accumulate) for lo, lg in zip(lora_layers, lora_grads_layers)]
    LA = (CLora * n)(*[p_[0] for p_ in pairs])
    LG = (CLoraGrads * n)(*[p_[1] for p_ in pairs])
    dg_final = torch.empty_like(g_final) if want_head else None
    dW_lm = torch.empty_like(W_lm) if want_head else None
    dX_embed = torch.empty_like(X_final)
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    need = L.alch_stack_backward_lora_workspace_bytes(C.byref(shape), n_layers, vocab, batch.total_tokens,
                                                      batch.max_seqlen, rank)
    ws = workspace if workspace is not None else _workspace(need, dev)
    hk = None
    if hooks is not None:
        ready, preempt = hooks
        hk = CHooks(HOOK_FN(ready) if ready else HOOK_FN(), HOOK_FN(preempt) if preempt else HOOK_FN(), None)
    _check(L.alch_stack_backward_lora(C.byref(shape), n_layers, vocab, C.byref(batch.c), SA, WA, LA, _ptr(X_final),
                                      _ptr(g_final), _ptr(W_lm), _ptr(labels), _ptr(loss_mask), GA, LG, _ptr(dg_final),
                                      _ptr(dW_lm), _ptr(dX_embed), _ptr(loss), C.byref(hk) if hk else None, _ptr(ws),
                                      ws.numel(), _stream_handle(stream)))
    layers = []
    for g, lg in zip(grads_layers, lora_grads_layers):
        d = dict(g)
        d.update(lg)
        layers.append(d)
    return dict(loss=loss, dX_embed=dX_embed, dg_final=dg_final, dW_lm=dW_lm, layers=layers)


class CDpo(C.Structure):
    _fields_ = [("n_items", C.c_int32), ("n_pairs", C.c_int32), ("item_row", C.c_void_p), ("item_label", C.c_void_p),
                ("item_slot", C.c_void_p), ("item_row_host", C.c_void_p), ("ref_logp", C.c_void_p), ("beta", C.c_float),
                ("z_out", C.c_void_p)]


class DpoItems:
    """The scored tokens of a DPO step, uploaded once: device copies of item_row / item_label / item_slot and of the
    reference sums, plus the host copy of item_row the library validates.  Pass it as `item_row` to
    alch_stack_backward_dpo (the other item arguments are then ignored) to keep the call free of host-to-device
    copies, e.g. under graph capture."""

    def __init__(self, item_row, item_label, item_slot, ref_logp, device="cuda"):
        self.rows_host = np.ascontiguousarray(item_row, dtype=np.int32)
        i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device)
        self.row, self.label, self.slot = i32(self.rows_host), i32(item_label), i32(item_slot)
        self.ref = ref_logp if torch.is_tensor(ref_logp) else \
            torch.from_numpy(np.ascontiguousarray(ref_logp, dtype=np.float32)).to(device)
        self.n_items, self.n_pairs = int(self.rows_host.shape[0]), int(self.ref.numel() // 2)
        self.z = torch.empty(max(self.n_pairs, 1), dtype=torch.float32, device=device)


def alch_stack_backward_dpo(shape, batch, saved_layers, weights_layers, X_final, g_final, W_lm, item_row, item_label,
                            item_slot, ref_logp, beta, lora_layers=None, rank=0, scale=1.0, want=WEIGHT_KEYS,
                            want_head=True, lora_grads_layers=None, grads_layers=None, accumulate=False, hooks=None,
                            workspace=None, stream=None):
    """Stack backward under the DPO loss.  item_row / item_label / item_slot: int32 numpy arrays, one entry per
    scored token, rows ascending; ref_logp: float32 [2 * n_pairs] (numpy or device tensor); or item_row = a DpoItems
    holding all four.  lora_layers: None, or
    per layer a dict projection -> (A, B).  Returns the dict of alch_stack_backward plus z (device [n_pairs])."""
    L = lib()
    dev = X_final.device
    n_layers = len(saved_layers)
    vocab = W_lm.shape[0]
    it = item_row if isinstance(item_row, DpoItems) else DpoItems(item_row, item_label, item_slot, ref_logp, dev)
    n_pairs, z = it.n_pairs, it.z
    dpo = CDpo(it.n_items, n_pairs, it.row.data_ptr(), it.label.data_ptr(), it.slot.data_ptr(), it.rows_host.ctypes.data,
               it.ref.data_ptr(), beta, z.data_ptr())
    if grads_layers is None:
        grads_layers = [{"d" + k: torch.empty_like(w[k]) for k in want} for w in weights_layers]
    n = max(n_layers, 1)
    SA = (CSaved * n)(*[_saved_struct(s_, 0) for s_ in saved_layers])
    WA = (CWeights * n)(*[_weights_struct(w, 0) for w in weights_layers])
    GA = (CWgrads * n)(*[_wgrads_struct(g, accumulate) for g in grads_layers])
    LA = LG = None
    if lora_layers is not None:
        if lora_grads_layers is None:
            lora_grads_layers = []
            for lo in lora_layers:
                g = {}
                for p_, (A_, B_) in lo.items():
                    g["dA" + p_], g["dB" + p_] = torch.empty_like(A_), torch.empty_like(B_)
                lora_grads_layers.append(g)
        pairs = [_lora_structs(lo, lg, rank, scale, accumulate) for lo, lg in zip(lora_layers, lora_grads_layers)]
        LA = (CLora * n)(*[p_[0] for p_ in pairs])
        LG = (CLoraGrads * n)(*[p_[1] for p_ in pairs])
        need = L.alch_stack_backward_lora_workspace_bytes(C.byref(shape), n_layers, vocab, batch.total_tokens,
                                                          batch.max_seqlen, rank)
    else:
        need = L.alch_stack_backward_workspace_bytes(C.byref(shape), n_layers, vocab, batch.total_tokens, batch.max_seqlen)
    dg_final = torch.empty_like(g_final) if want_head else None
    dW_lm = torch.empty_like(W_lm) if want_head else None
    dX_embed = torch.empty_like(X_final)
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    ws = workspace if workspace is not None else _workspace(need, dev)
    hk = None
    if hooks is not None:
        ready, preempt = hooks
        hk = CHooks(HOOK_FN(ready) if ready else HOOK_FN(), HOOK_FN(preempt) if preempt else HOOK_FN(), None)
    _check(L.alch_stack_backward_dpo(C.byref(shape), n_layers, vocab, C.byref(batch.c), SA, WA, LA, _ptr(X_final),
                                     _ptr(g_final), _ptr(W_lm), C.byref(dpo), GA, LG, _ptr(dg_final), _ptr(dW_lm),
                                     _ptr(dX_embed), _ptr(loss), C.byref(hk) if hk else None, _ptr(ws), ws.numel(),
                                     _stream_handle(stream)))
    layers = []
    for i, g in enumerate(grads_layers):
        d = dict(g)
        if lora_grads_layers is not None:
            d.update(lora_grads_layers[i])
        layers.append(d)
    return dict(loss=loss, z=z[:n_pairs], dX_embed=dX_embed, dg_final=dg_final, dW_lm=dW_lm, layers=layers)


def alch_gemm(M, N, terms, a_kmajor, b_kmajor, out=None, accumulate=False, stream=None, workspace=None):
    """terms: list of (A, B, K) device tensors (2-D, last dim contiguous).  Returns C [M, N].  workspace: optional
    uint8 device tensor of lib().alch_gemm_workspace_bytes() bytes (lets the last round of tiles be split)."""
    L = lib()
    A0 = terms[0][0]
    code = ALCH_BF16 if A0.dtype == torch.bfloat16 else ALCH_F32
    if out is None:
        out = torch.empty((M, N), dtype=A0.dtype, device=A0.device)
    arr = (CGemmTerm * len(terms))(*[CGemmTerm(a.data_ptr(), b.data_ptr(), k, a.stride(0), b.stride(0))
                                     for a, b, k in terms])
    _check(L.alch_gemm_ws(code, M, N, 1 if a_kmajor else 0, 1 if b_kmajor else 0, len(terms), arr, _ptr(out),
                          out.stride(0), 1 if accumulate else 0, _ptr(workspace),
                          0 if workspace is None else workspace.numel(), _stream_handle(stream)))
    return out


def alch_attention_forward(shape, batch, Q, K, V, stream=None):
    """Returns (O, LSE) of causal grouped-query attention over post-RoPE Q, K and V."""
    L = lib()
    O = torch.empty_like(Q)
    LSE = torch.empty((Q.shape[0], shape.n_q_heads), dtype=torch.float32, device=Q.device)
    _check(L.alch_attention_forward(C.byref(shape), C.byref(batch.c), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE),
                                    _stream_handle(stream)))
    return O, LSE


def alch_trace_enable(on):
    _check(lib().alch_trace_enable(1 if on else 0))


def alch_trace_collect(max_records=65536):
    """Returns a list of (kind name, flops, bytes, ms) in launch order (waits for the launches)."""
    buf = (CTraceRecord * max_records)()
    n = C.c_int32(0)
    _check(lib().alch_trace_collect(buf, max_records, C.byref(n)))
    return [(TRACE_KINDS[buf[i].kind], buf[i].flops, buf[i].bytes, buf[i].ms) for i in range(n.value)]
