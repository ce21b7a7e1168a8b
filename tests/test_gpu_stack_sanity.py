"""Two sanity bands on the stack at the bench's own sizes (8 x 4096 tokens, vocabulary 128,256, Llama-3-8B-shaped
layers, a reduced layer count), through the code path bench.py times:
  - the cross-entropy of a randomly initialised model: with logits of variance s^2 (here 0.02^2 * hidden, the
    final norm has unit gain) the expected loss is ln V + s^2 / 2;
  - the paper's Section 1 / Section 6 ratio: an iteration that recomputes the forward pass costs between 1.26 and
    1.75 times one that starts from the saved activations (forward = 30-43 % of an iteration).
Neither is parity; both would catch a mis-scaled loss or a backward that silently skips work."""
import argparse
import math

import pytest

pytestmark = pytest.mark.gpu


def test_random_init_loss_and_reuse_over_recompute_ratio():
    import torch
    import bench
    import paper_2503_01066_amd as A
    args = argparse.Namespace(workload="config4", layers=8, steps=2, warmup=1, lora_rank=0, frozen_base=False, loss_mask=False,
                              offload=False, six_stream=False, four_stream=False)
    res = bench.run_config4(args, torch, A)
    V, H = 128256, 4096
    expected = math.log(V) + 0.5 * 0.02 ** 2 * H
    print("loss %.4f expected %.4f; reuse %.1f ms, ratio %.3f" % (res["loss"], expected, res["ms_per_step"],
                                                                 res["reuse_speedup_over_recompute"]), flush=True)
    assert abs(res["loss"] - expected) <= 0.05 * expected
    assert abs(res["loss_expected_random_init"] - expected) < 1e-9
    assert 1.26 <= res["reuse_speedup_over_recompute"] <= 1.75
