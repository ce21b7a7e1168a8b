"""GPU parity of the shared-prefix path (Section 4.1 of the paper, preference alignment: responses attend to
the saved KV cache of their prompt; chosen and rejected share it) against the fp64 oracle:
attention forward, layer backward, and the forward over the response rows alone."""
import numpy as np
import pytest
import torch

import synth_inputs as synth
from helpers import TOL, to_dev, to_np, f64, rel_err, cosine, oracle_shape, alch_shape
from oracle import WEIGHT_KEYS
from oracle.prefix import layer_forward_prefix, layer_backward_reuse_prefix

pytestmark = pytest.mark.gpu
REC = ("X", "X2", "Q", "K", "V", "O", "G", "U")

# (dtype, shape, prompt lengths, response lengths per prompt): f32 / head_dim 8 and bf16 / head_dim 64 take the
# plain kernels, bf16 / head_dim 128 the matrix-core kernels (prompts and responses spanning several 64- and
# 128-row tiles, ragged tails, a prompt without responses, an empty response, three responses on one prompt)
CASES = [("f32", "tiny", [4, 2, 3], [[3, 2], [1, 4], []]),
         ("bf16", "medium64", [130, 61], [[40, 75], [20, 20]]),
         ("bf16", "medium", [300, 65, 128], [[70, 129], [1, 0, 200], []]),
         ("bf16", "medium", [257], [[64, 64]]),
         ("bf16", "medium", [31, 700], [[300, 10], [5, 140]])]


def make(dtype, shape_name, prompts, responses, seed):
    shp = synth.shape_dict(shape_name)
    osh = oracle_shape(shp)
    b = synth.preference_batch(prompts, responses, 100, seed)
    T = int(b["cu"][-1])
    W = synth.layer_weights(shp, seed, dtype, std=0.3 if shape_name == "tiny" else 0.02, gain_std=0.1)
    X = synth.activations(T, shp["hidden"], seed + 1, dtype)
    Y64, rec64 = layer_forward_prefix(osh, b["cu"], b["prefix"], X.astype(np.float64), f64(W))
    rec = {k: synth.quantize(rec64[k].astype(np.float32), dtype) for k in REC}
    rec["LSE"] = rec64["LSE"].astype(np.float32)
    dY = synth.activations(T, shp["hidden"], seed + 2, dtype, std=1.0 if dtype == "f32" else 0.01)
    return shp, osh, b, W, X, Y64, rec64, rec, dY


def dev_record(rec, dtype):
    d = {k: to_dev(rec[k], dtype) for k in REC}
    d["LSE"] = torch.from_numpy(rec["LSE"]).cuda()
    return d


@pytest.mark.parametrize("dtype,shape_name,prompts,responses", CASES)
def test_layer_backward_with_shared_prefixes(dtype, shape_name, prompts, responses):
    import paper_2503_01066_amd as A
    shp, osh, b, W, X, _, _, rec, dY = make(dtype, shape_name, prompts, responses, 5)
    ref = layer_backward_reuse_prefix(osh, b["cu"], b["prefix"], f64(rec), f64(W), dY)
    batch = A.Batch(b["cu"], positions=b["positions"], prefix=b["prefix"])
    out = A.alch_layer_backward(alch_shape(shp, dtype), batch, dev_record(rec, dtype),
                                {k: to_dev(v, dtype) for k, v in W.items()}, to_dev(dY, dtype))
    torch.cuda.synchronize()
    for k in ["dX"] + ["d" + w for w in WEIGHT_KEYS]:
        g = to_np(out[k])
        assert np.isfinite(g).all(), k
        assert rel_err(g, ref[k]) <= TOL[dtype], (k, rel_err(g, ref[k]), cosine(g, ref[k]))
    # the prompt rows alone, too: their gradient comes through the shared keys and values
    n_p = int(b["cu"][b["n_prompts"]])
    assert rel_err(to_np(out["dX"])[:n_p], ref["dX"][:n_p]) <= TOL[dtype]


@pytest.mark.parametrize("dtype,shape_name,prompts,responses", CASES)
def test_forward_over_the_responses_alone(dtype, shape_name, prompts, responses):
    # rows of the prompts: given (what serving left behind); rows of the responses: computed by the library
    import paper_2503_01066_amd as A
    shp, osh, b, W, X, Y64, rec64, rec, _ = make(dtype, shape_name, prompts, responses, 9)
    n_p = int(b["cu"][b["n_prompts"]])
    T = int(b["cu"][-1])
    batch = A.Batch(b["cu"], positions=b["positions"], prefix=b["prefix"])
    drec = dev_record(rec, dtype)
    marker = 7.0
    for k in drec:                       # response rows start out as a marker value
        drec[k][n_p:] = marker
    Y = torch.full((T, shp["hidden"]), marker, dtype=drec["X"].dtype, device="cuda")
    A.alch_layer_forward(alch_shape(shp, dtype), batch, to_dev(X, dtype), {k: to_dev(v, dtype) for k, v in W.items()},
                         seq_begin=b["n_prompts"], rec=drec, Y=Y)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    for k in REC + ("LSE",):
        got = to_np(drec[k])
        want = np.asarray(rec[k], dtype=np.float64)
        assert np.array_equal(got[:n_p], want[:n_p]), k          # prompt rows untouched
        if T > n_p:
            assert rel_err(got[n_p:], rec64[k][n_p:]) <= tol, (k, rel_err(got[n_p:], rec64[k][n_p:]))
    assert np.all(to_np(Y)[:n_p] == marker)
    if T > n_p:
        assert rel_err(to_np(Y)[n_p:], Y64[n_p:]) <= tol


def test_whole_batch_forward_with_prefixes_equals_the_oracle():
    import paper_2503_01066_amd as A
    dtype = "bf16"
    shp, osh, b, W, X, Y64, rec64, rec, _ = make(dtype, "medium", [200, 90], [[100, 30], [64, 65]], 13)
    batch = A.Batch(b["cu"], positions=b["positions"], prefix=b["prefix"])
    Y, drec = A.alch_layer_forward(alch_shape(shp, dtype), batch, to_dev(X, dtype), {k: to_dev(v, dtype) for k, v in W.items()})
    torch.cuda.synchronize()
    assert rel_err(to_np(Y), Y64) <= TOL[dtype]
    for k in REC + ("LSE",):
        assert rel_err(to_np(drec[k]), rec64[k]) <= TOL[dtype], k
