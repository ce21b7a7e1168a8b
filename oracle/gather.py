"""Oracle for capture/pack: stable gather of the rows a keep-mask selects.

Test infrastructure only (see the package docstring).

Paper basis: Section 4.1 (only prefill tokens are recorded), Section 5 (each saved
tensor is recorded per layer).  The per-token keep mask generalises "record this
token or not"; the result is the unique ascending-order gather, so the oracle is
the definition itself.
"""
import numpy as np


def gather_pack(mask, cu_seqlens, streams):
    """mask: uint8 [T], any nonzero value keeps the token.
    cu_seqlens: int [n_seqs+1], cu[0] = 0, non-decreasing, cu[-1] = T.
    streams: list of 2-D arrays [T, width_k] (any dtype; rows are copied bit-for-bit).

    Returns (kept_index int32 [n_kept] ascending, cu_kept int32 [n_seqs+1],
             packed list of arrays [n_kept, width_k]).
    cu_kept[s] = number of kept tokens t with t < cu_seqlens[s].
    """
    mask = np.asarray(mask)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    T = mask.shape[0]
    assert cu[0] == 0 and cu[-1] == T and np.all(np.diff(cu) >= 0)
    kept = np.array([t for t in range(T) if mask[t] != 0], dtype=np.int32)
    cu_kept = np.array([int(np.sum(kept < c)) for c in cu], dtype=np.int32)
    packed = []
    for src in streams:
        src = np.asarray(src)
        assert src.shape[0] == T
        dst = np.empty((kept.shape[0],) + src.shape[1:], dtype=src.dtype)
        for r, t in enumerate(kept):
            dst[r] = src[t]
        packed.append(dst)
    return kept, cu_kept, packed
