"""alch_capture_pack_static (the entry point that neither takes nor allocates a workspace) against
alch_capture_pack and the gather oracle: two calls in a row on the same output buffers, the second on a
smaller batch, so that whatever the first call left in the library's built-in scratch is still there, and a third
on a batch small enough for the single-launch scan."""
import numpy as np
import pytest
import torch

import synth_inputs as synth
from oracle import gather_pack

pytestmark = pytest.mark.gpu


def _case(lens, keep, seed, widths):
    rng = np.random.default_rng(seed)
    cu = synth.ragged_cu(lens)
    T = int(cu[-1])
    mask = synth.keep_mask(T, keep, seed + 1)
    srcs = [rng.integers(0, 65535, size=(T, w)).astype(np.uint16) for w in widths]
    return cu, T, mask, srcs


def test_static_scratch_matches_workspace_call_twice_in_a_row():
    import paper_2503_01066_amd as A
    # (batches of up to 262,144 tokens are scanned by a single launch that needs no scratch: the first two cases
    # are larger, so their block counters do live in the built-in array; the third takes the single-launch scan)
    widths = (8, 8, 24)
    big = _case([150000, 0, 170100, 1, 50000, 777], 0.4, 0, widths)   # 91 scan blocks, ragged tail
    small = _case([130000, 61, 0, 140200], 0.7, 5, widths)            # fewer blocks than the call before
    tiny = _case([130, 61, 0, 200], 0.7, 7, widths)
    cap = big[1]
    # caller-owned outputs, allocated once and reused by both calls (the entry point itself allocates nothing)
    kept = torch.empty(cap, dtype=torch.int32, device="cuda")
    status = torch.empty(2, dtype=torch.int32, device="cuda")
    dsts = [torch.empty((cap, w), dtype=torch.int16, device="cuda") for w in widths]
    for cu, T, mask, srcs in (big, small, tiny):
        batch = A.Batch(cu)
        dmask = torch.from_numpy(mask).cuda()
        wide = torch.zeros((T, 40), dtype=torch.int16, device="cuda")   # third stream: column slice of a fused buffer
        wide[:, 8:32] = torch.from_numpy(srcs[2].view(np.int16)).cuda()
        devs = [torch.from_numpy(srcs[0].view(np.int16)).cuda(), torch.from_numpy(srcs[1].view(np.int16)).cuda(),
                wide[:, 8:32]]
        cu_kept = torch.empty(batch.n_seqs + 1, dtype=torch.int32, device="cuda")
        for t in [kept, status, cu_kept] + dsts:
            t.fill_(-1)
        A.alch_capture_pack_static(batch, dmask, devs, dsts, kept, cu_kept, status)
        r_kept, r_cu, r_status, r_dsts = A.alch_capture_pack(batch, dmask, devs, capacity=cap)
        torch.cuda.synchronize()
        ok, ocu, opacked = gather_pack(mask, cu, srcs)
        n = len(ok)
        assert status.cpu().tolist() == [n, 0] == r_status.cpu().tolist()
        assert np.array_equal(kept[:n].cpu().numpy(), r_kept[:n].cpu().numpy())
        assert np.array_equal(kept[:n].cpu().numpy(), ok)
        assert np.array_equal(cu_kept.cpu().numpy(), r_cu.cpu().numpy()) and np.array_equal(r_cu.cpu().numpy(), ocu)
        for d, r, o in zip(dsts, r_dsts, opacked):
            assert torch.equal(d[:n], r[:n])
            assert np.array_equal(d[:n].cpu().numpy().view(np.uint8), o.view(np.uint8))
            assert bool((d[n:] == -1).all())                            # nothing written beyond the kept rows


def test_static_scratch_empty_batch_and_overflow_flag():
    import paper_2503_01066_amd as A
    cu, T, mask, srcs = _case([50, 50], 1.0, 3, (16,))
    batch = A.Batch(cu)
    kept = torch.full((30,), -1, dtype=torch.int32, device="cuda")
    status = torch.empty(2, dtype=torch.int32, device="cuda")
    cu_kept = torch.empty(3, dtype=torch.int32, device="cuda")
    dst = torch.empty((30, 16), dtype=torch.int16, device="cuda")
    A.alch_capture_pack_static(batch, torch.from_numpy(mask).cuda(), [torch.from_numpy(srcs[0].view(np.int16)).cuda()],
                               [dst], kept, cu_kept, status)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [100, 1]
    assert np.array_equal(kept.cpu().numpy(), np.arange(30))
    assert np.array_equal(dst.cpu().numpy().view(np.uint16), srcs[0][:30])
    empty = A.Batch(np.zeros(1, np.int32))
    cu0 = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    A.alch_capture_pack_static(empty, torch.zeros(0, dtype=torch.uint8, device="cuda"), [], [], kept[:0], cu0, status)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, 0] and cu0.cpu().tolist() == [0]
