"""Pins for the capture/pack oracle: brute force on tiny inputs, closed-form sizes,
degenerate masks (Section 4.1: which tokens are recorded; Section 4.3.1: the size of
what is recorded depends only on the number of tokens)."""
import numpy as np
import pytest
from oracle import gather_pack


def brute(mask, cu, streams):
    kept = []
    for t in range(len(mask)):
        if mask[t]:
            kept.append(t)
    cu_kept = []
    for c in cu:
        n = 0
        for t in kept:
            if t < c:
                n += 1
        cu_kept.append(n)
    outs = []
    for s in streams:
        rows = []
        for t in kept:
            rows.append([s[t][j] for j in range(s.shape[1])])
        outs.append(rows)
    return kept, cu_kept, outs


@pytest.mark.parametrize("seed", range(6))
def test_gather_matches_brute_force(seed):
    rng = np.random.default_rng(seed)
    lens = rng.integers(0, 6, size=5)          # includes empty and single-token sequences
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    mask = (rng.random(T) < 0.5).astype(np.uint8) * rng.integers(1, 255, size=T).astype(np.uint8)
    a = rng.integers(0, 2 ** 16, size=(T, 3)).astype(np.uint16)
    wide = rng.standard_normal((T, 10)).astype(np.float32)
    b = wide[:, 2:7]                           # strided view of a wider buffer
    kept, cu_kept, (pa, pb) = gather_pack(mask, cu, [a, b])
    bk, bcu, (ba, bb) = brute(mask, cu, [a, b])
    assert kept.tolist() == bk
    assert cu_kept.tolist() == bcu
    assert pa.tolist() == ba
    assert pb.view(np.uint32).tolist() == np.array(bb, dtype=np.float32).reshape(-1, 5).view(np.uint32).tolist() if bk else pb.shape[0] == 0


def test_gather_degenerate_masks_and_sizes():
    cu = np.array([0, 3, 3, 4, 9], dtype=np.int32)
    T = 9
    src = np.arange(T * 4, dtype=np.int32).reshape(T, 4)
    lse = np.arange(T * 2, dtype=np.float32).reshape(T, 2)
    for mask in (np.zeros(T, np.uint8), np.ones(T, np.uint8), np.eye(1, T, 4, dtype=np.uint8)[0]):
        kept, cu_kept, (p, q) = gather_pack(mask, cu, [src, lse])
        n = int(np.count_nonzero(mask))
        assert kept.shape == (n,) and p.shape == (n, 4) and q.shape == (n, 2)
        # closed form: packed bytes = n_kept * sum of row bytes
        assert p.nbytes + q.nbytes == n * (4 * 4 + 2 * 4)
        assert cu_kept[0] == 0 and cu_kept[-1] == n
        assert np.all(np.diff(cu_kept) == [np.count_nonzero(mask[cu[s]:cu[s + 1]]) for s in range(4)])
        assert np.array_equal(p, src[mask != 0])
    kept, _, _ = gather_pack(np.ones(T, np.uint8), cu, [src])
    assert kept.tolist() == list(range(T))      # keep-all is the identity
