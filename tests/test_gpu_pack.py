"""GPU parity of capture/pack against the gather oracle: bit-exact indices and rows."""
import numpy as np
import pytest
import torch

import synth_inputs as synth
from oracle import gather_pack

pytestmark = pytest.mark.gpu


def run_pack(cu, mask, srcs_np, capacity=None, strided=False):
    import paper_2503_01066_amd as A
    batch = A.Batch(cu)
    dev_mask = torch.from_numpy(mask).cuda()
    streams = []
    for s in srcs_np:
        t = torch.from_numpy(s).cuda()
        if strided:  # place the stream as a column slice of a wider fused buffer
            pad = 8 if s.dtype.itemsize == 2 else 4
            wide = torch.zeros((s.shape[0], s.shape[1] + 2 * pad), dtype=t.dtype, device="cuda")
            wide[:, pad:pad + s.shape[1]] = t
            t = wide[:, pad:pad + s.shape[1]]
        streams.append(t)
    kept, cu_kept, status, dsts = A.alch_capture_pack(batch, dev_mask, streams, capacity=capacity)
    torch.cuda.synchronize()
    return kept.cpu().numpy(), cu_kept.cpu().numpy(), status.cpu().numpy(), [d.cpu().numpy() for d in dsts]


def check(cu, mask, srcs_np, strided=False):
    ok, ocu, opacked = gather_pack(mask, cu, srcs_np)
    kept, cu_kept, status, dsts = run_pack(cu, mask, srcs_np, strided=strided)
    n = len(ok)
    assert status[0] == n and status[1] == 0
    assert np.array_equal(kept[:n], ok)
    assert np.array_equal(cu_kept, ocu)
    for d, o in zip(dsts, opacked):
        assert np.array_equal(d[:n].view(np.uint8), o.view(np.uint8))


def streams_for(T, rng, widths=(24, 8, 40), dtype=np.uint16):
    return [rng.integers(0, np.iinfo(dtype).max, size=(T, w)).astype(dtype) for w in widths]


@pytest.mark.parametrize("seed", range(4))
def test_tiny_ragged(seed):
    rng = np.random.default_rng(seed)
    lens = rng.integers(0, 7, size=6)
    cu = synth.ragged_cu(lens)
    T = int(cu[-1])
    mask = (rng.random(T) < 0.5).astype(np.uint8) * rng.integers(1, 255, size=T).astype(np.uint8)
    check(cu, mask, streams_for(T, rng))


def test_degenerate_masks_and_empty_batch():
    rng = np.random.default_rng(5)
    cu = synth.ragged_cu([3, 0, 1, 5])
    for mask in (np.zeros(9, np.uint8), np.ones(9, np.uint8)):
        check(cu, mask, streams_for(9, rng))
    check(np.zeros(1, np.int32), np.zeros(0, np.uint8), [np.zeros((0, 8), np.uint16)])
    check(synth.ragged_cu([0, 0]), np.zeros(0, np.uint8), [np.zeros((0, 8), np.uint16)])


def test_config1_record_streams_fp32():
    # config 1: B=2 x S=128, hidden 256, 4 heads x 64, FFN 1024, fp32; mask ~ Bernoulli(0.5), seed 0
    rng = np.random.default_rng(0)
    cu = synth.uniform_cu(2, 128)
    mask = synth.keep_mask(256, 0.5, 0)
    widths = dict(X=256, X2=256, Q=256, K=256, V=256, O=256, G=1024, U=1024, LSE=4)
    srcs = [rng.standard_normal((256, w)).astype(np.float32) for w in widths.values()]
    check(cu, mask, srcs)
    check(cu, mask, srcs, strided=True)


def test_many_blocks_ragged_tail_and_odd_widths():
    # spans several 4096-token scan blocks with a ragged tail; widths that are not multiples of 16 bytes
    rng = np.random.default_rng(1)
    lens = synth.random_lengths(7, 256, 4096, 3)
    cu = synth.ragged_cu(lens)
    T = int(cu[-1])
    mask = synth.keep_mask(T, 0.25, 4)
    srcs = streams_for(T, rng, widths=(64, 8, 6, 130))      # 6 and 130 uint16 -> 12 / 260 byte rows (4-byte path)
    check(cu, mask, srcs)
    check(cu, mask, streams_for(T, rng, widths=(64, 512)), strided=True)
    # exactly a multiple of the scan block, all kept
    cu2 = synth.uniform_cu(2, 4096)
    check(cu2, np.ones(8192, np.uint8), streams_for(8192, rng, widths=(8,)))


def test_batches_beyond_the_single_launch_scan():
    # up to 262,144 tokens the mask scan is one single-work-group launch; beyond that the four-kernel scan with block
    # counts in the workspace runs: both sides of the limit, ragged, with empty sequences and a boundary inside a chunk
    rng = np.random.default_rng(6)
    for lens, keep in (([150000, 0, 112143, 1], 0.3), ([262144], 0.5), ([200000, 62145], 0.1), ([300001, 7, 0, 123457], 0.25)):
        cu = synth.ragged_cu(lens)
        T = int(cu[-1])
        mask = synth.keep_mask(T, keep, 8)
        check(cu, mask, streams_for(T, rng, widths=(8, 2)))


def test_more_streams_than_one_launch_takes():
    rng = np.random.default_rng(2)
    cu = synth.ragged_cu([100, 37])
    mask = synth.keep_mask(137, 0.4, 1)
    check(cu, mask, streams_for(137, rng, widths=tuple([8] * 37)))


def test_capacity_overflow_is_flagged_and_bounded():
    rng = np.random.default_rng(3)
    cu = synth.ragged_cu([50, 50])
    mask = np.ones(100, np.uint8)
    srcs = streams_for(100, rng, widths=(16,))
    kept, cu_kept, status, dsts = run_pack(cu, mask, srcs, capacity=30)
    assert status[0] == 100 and status[1] == 1
    assert np.array_equal(kept[:30], np.arange(30))
    assert np.array_equal(dsts[0][:30], srcs[0][:30])


def test_deterministic_bits():
    rng = np.random.default_rng(4)
    cu = synth.ragged_cu([3000, 2000, 4100])
    mask = synth.keep_mask(9100, 0.25, 9)
    srcs = streams_for(9100, rng, widths=(256,))
    a = run_pack(cu, mask, srcs)
    b = run_pack(cu, mask, srcs)
    n = a[2][0]
    assert np.array_equal(a[0][:n], b[0][:n]) and np.array_equal(a[3][0][:n], b[3][0][:n])


@pytest.mark.parametrize("keep,capacity", [(0.3, None), (0.0, None), (1.0, None), (0.6, 1000)])
def test_gather_with_the_index_of_an_earlier_pack(keep, capacity):
    # one scan per batch, one gather per layer: the streams of a second "layer" are gathered with the index the
    # first call left on the device; bit-exact against the oracle on those streams, also when the capacity cuts
    import paper_2503_01066_amd as A
    rng = np.random.default_rng(17)
    cu = synth.ragged_cu([700, 0, 3000, 1, 513])
    T = int(cu[-1])
    mask = synth.keep_mask(T, keep, 2)
    first, second = streams_for(T, rng, widths=(64,)), streams_for(T, rng, widths=(24, 8, 520))
    batch = A.Batch(cu)
    kept, cu_kept, status, _ = A.alch_capture_pack(batch, torch.from_numpy(mask).cuda(), [torch.from_numpy(s).cuda() for s in first],
                                                   capacity=capacity)
    wide = torch.zeros((T, 600), dtype=torch.int16, device="cuda")          # one stream as a column slice
    wide[:, 40:560] = torch.from_numpy(second[2].view(np.int16)).cuda()
    devs = [torch.from_numpy(second[0].view(np.int16)).cuda(), torch.from_numpy(second[1].view(np.int16)).cuda(), wide[:, 40:560]]
    dsts = A.alch_capture_gather(batch, kept, status, devs, capacity=capacity)
    torch.cuda.synchronize()
    ok, _, opacked = gather_pack(mask, cu, second)
    n = len(ok) if capacity is None else min(len(ok), capacity)
    assert int(status[0]) == len(ok) and int(status[1]) == (0 if capacity is None or len(ok) <= capacity else 1)
    for d, o in zip(dsts, opacked):
        assert np.array_equal(d[:n].cpu().numpy().view(np.uint8), o[:n].view(np.uint8))
