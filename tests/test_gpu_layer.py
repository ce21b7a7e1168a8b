"""GPU parity of alch_layer_backward against the fp64 oracle on the same seeded inputs.
Bar: per output tensor max|gpu - oracle| / max|oracle| <= 2e-2 (bf16) / 1e-4 (f32)."""
import numpy as np
import pytest
import torch

import synth_inputs as synth
from helpers import TOL, to_dev, to_np, f64, rel_err, cosine, oracle_shape, alch_shape
from oracle import layer_forward, layer_backward_reuse, attention_lse, WEIGHT_KEYS

pytestmark = pytest.mark.gpu
REC = ("X", "X2", "Q", "K", "V", "O", "G", "U")


def make_case(shape_name, dtype, cu, seed, record, wstd=0.02, dy_std=1.0, gain_std=0.1):
    shp = synth.shape_dict(shape_name)
    osh = oracle_shape(shp)
    T = int(cu[-1])
    W = synth.layer_weights(shp, seed, dtype, std=wstd, gain_std=gain_std)
    if record == "forward":
        X = synth.activations(T, shp["hidden"], seed + 1, dtype)
        _, rec64 = layer_forward(osh, cu, None, X.astype(np.float64), f64(W))
        rec = {k: synth.quantize(rec64[k].astype(np.float32), dtype) for k in REC}
        rec["LSE"] = rec64["LSE"].astype(np.float32)
    else:
        rec = synth.drawn_record(shp, T, seed + 1, dtype)
        rec["LSE"] = attention_lse(osh, cu, rec["Q"].astype(np.float64), rec["K"].astype(np.float64)).astype(np.float32)
    dY = synth.activations(T, shp["hidden"], seed + 2, dtype, std=dy_std)
    return shp, osh, W, rec, dY


def run_gpu(shp, dtype, cu, W, rec, dY, loss_mask=None, want=WEIGHT_KEYS, positions=None, **kw):
    import paper_2503_01066_amd as A
    batch = A.Batch(cu, positions=positions)
    dW = {k: to_dev(v, dtype) for k, v in W.items()}
    drec = {k: to_dev(rec[k], dtype) for k in REC}
    drec["LSE"] = torch.from_numpy(rec["LSE"]).cuda()
    dm = None if loss_mask is None else torch.from_numpy(loss_mask).cuda()
    out = A.alch_layer_backward(alch_shape(shp, dtype), batch, drec, dW, to_dev(dY, dtype), loss_mask=dm, want=want, **kw)
    torch.cuda.synchronize()
    return {k: to_np(v) for k, v in out.items()}


def compare(gpu, ref, dtype, keys=None):
    worst = {}
    for k in (keys or gpu.keys()):
        e = rel_err(gpu[k], ref[k])
        worst[k] = e
        assert np.isfinite(gpu[k]).all(), k
        assert e <= TOL[dtype], (k, e, cosine(gpu[k], ref[k]))
    return worst


def test_config1_fp32_layer_with_loss_mask():
    # config 1: fp32, hidden 256, 4x64 MHA, FFN 1024, eps 1e-6, base 1e4, B=2 x S=128, record from a forward
    cu = synth.uniform_cu(2, 128)
    shp, osh, W, rec, dY = make_case("config1", "f32", cu, 0, "forward", gain_std=0.0)
    mask = synth.keep_mask(256, 0.5, 0)
    for lm in (None, mask):
        ref = layer_backward_reuse(osh, cu, None, f64(rec), f64(W), dY, lm)
        gpu = run_gpu(shp, "f32", cu, W, rec, dY, loss_mask=lm)
        compare(gpu, ref, "f32")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_tiny_ragged_gqa(dtype):
    cu = synth.ragged_cu([1, 5, 0, 8, 3])
    shp, osh, W, rec, dY = make_case("tiny", dtype, cu, 3, "forward", wstd=0.3)
    ref = layer_backward_reuse(osh, cu, None, f64(rec), f64(W), dY)
    compare(run_gpu(shp, dtype, cu, W, rec, dY), ref, dtype)


@pytest.mark.parametrize("shape_name,lens", [("medium", [300, 1, 257, 64]), ("medium64", [130, 200, 77]),
                                             ("medium", [715, 128, 33])])
def test_medium_bf16_several_tiles_and_ragged_tail(shape_name, lens):
    # T is not a multiple of any tile size; several 256-wide tiles in every GEMM dimension
    cu = synth.ragged_cu(lens)
    for record in ("drawn", "forward"):
        shp, osh, W, rec, dY = make_case(shape_name, "bf16", cu, 5, record, dy_std=0.01)
        ref = layer_backward_reuse(osh, cu, None, f64(rec), f64(W), dY)
        compare(run_gpu(shp, "bf16", cu, W, rec, dY), ref, "bf16")


def test_loss_mask_positions_and_frozen_weights_bf16():
    cu = synth.ragged_cu([200, 313])
    T = 513
    shp, osh, W, rec, dY = make_case("medium", "bf16", cu, 7, "drawn", dy_std=0.01)
    mask = synth.keep_mask(T, 0.25, 1)
    pos = np.random.default_rng(2).integers(0, 3000, T).astype(np.int32)
    ref = layer_backward_reuse(osh, cu, pos, f64(rec), f64(W), dY, mask)
    gpu = run_gpu(shp, "bf16", cu, W, rec, dY, loss_mask=mask, positions=pos, want=("Wq", "Wd", "g2"))
    assert set(gpu) == {"dX", "dWq", "dWd", "dg2"}
    compare(gpu, ref, "bf16")


def test_accumulate_adds_to_existing_gradients():
    cu = synth.ragged_cu([100, 156])
    shp, osh, W, rec, dY = make_case("medium", "bf16", cu, 9, "drawn", dy_std=0.01)
    ref = layer_backward_reuse(osh, cu, None, f64(rec), f64(W), dY)
    base = {"d" + k: synth.quantize(0.5 * np.abs(ref["d" + k]).max() *
                                    np.random.default_rng(3).standard_normal(W[k].shape).astype(np.float32), "bf16")
            for k in WEIGHT_KEYS}
    grads = {k: to_dev(v, "bf16") for k, v in base.items()}
    gpu = run_gpu(shp, "bf16", cu, W, rec, dY, grads=grads, accumulate=True)
    want = {k: ref[k] + base[k] for k in base}
    want["dX"] = ref["dX"]
    compare(gpu, want, "bf16")


def test_empty_batch_and_stale_record():
    import paper_2503_01066_amd as A
    cu = np.zeros(1, np.int32)
    shp, osh, W, rec, dY = make_case("tiny", "f32", cu, 1, "drawn")
    gpu = run_gpu(shp, "f32", cu, W, rec, dY)
    for k in WEIGHT_KEYS:
        assert np.all(gpu["d" + k] == 0), k
    cu = synth.ragged_cu([4])
    shp, osh, W, rec, dY = make_case("tiny", "f32", cu, 1, "forward")
    with pytest.raises(A.AlchError) as e:
        run_gpu(shp, "f32", cu, W, rec, dY, saved_version=3, weights_version=4)
    assert e.value.code == -4


@pytest.mark.parametrize("dtype,shape_name,lens", [("f32", "tiny", [1, 5, 0, 8, 3]), ("bf16", "medium", [300, 1, 257, 64]),
                                                   ("bf16", "medium64", [130, 200, 77])])
def test_six_stream_record_is_completed_on_the_device(dtype, shape_name, lens):
    # the record of the capture workload (X, Q, K, V, G, U only): O, LSE and X2 are recomputed by the library;
    # the oracle completes the same rounded six tensors in fp64
    from oracle import complete_record
    cu = synth.ragged_cu(lens)
    shp, osh, W, rec, dY = make_case(shape_name, dtype, cu, 17, "forward", wstd=0.3 if shape_name == "tiny" else 0.02,
                                     dy_std=1.0 if dtype == "f32" else 0.01)
    six = {k: rec[k] for k in ("X", "Q", "K", "V", "G", "U")}
    ref = layer_backward_reuse(osh, cu, None, complete_record(osh, cu, f64(six), f64(W)), f64(W), dY)
    import paper_2503_01066_amd as A
    out = A.alch_layer_backward(alch_shape(shp, dtype), A.Batch(cu), {k: to_dev(v, dtype) for k, v in six.items()},
                                {k: to_dev(v, dtype) for k, v in W.items()}, to_dev(dY, dtype))
    torch.cuda.synchronize()
    compare({k: to_np(v) for k, v in out.items()}, ref, dtype)
    # only X2 missing: O and LSE are taken as saved
    part = {k: rec[k] for k in rec if k != "X2"}
    ref2 = layer_backward_reuse(osh, cu, None, complete_record(osh, cu, {k: np.asarray(v, dtype=np.float64) for k, v in part.items()}, f64(W)), f64(W), dY)
    d = {k: to_dev(v, dtype) for k, v in part.items() if k != "LSE"}
    d["LSE"] = torch.from_numpy(rec["LSE"]).cuda()
    out2 = A.alch_layer_backward(alch_shape(shp, dtype), A.Batch(cu), d, {k: to_dev(v, dtype) for k, v in W.items()},
                                 to_dev(dY, dtype))
    torch.cuda.synchronize()
    compare({k: to_np(v) for k, v in out2.items()}, ref2, dtype)


@pytest.mark.parametrize("dtype,shape_name,lens,keep", [("f32", "tiny", [1, 5, 0, 8, 3], None), ("bf16", "medium", [300, 1, 257, 64], None),
                                                        ("bf16", "medium", [300, 1, 257, 64], 0.3), ("f32", "tiny", [4, 9], 0.5),
                                                        ("bf16", "medium64", [130, 200, 77], None)])
def test_four_stream_record_is_completed_on_the_device(dtype, shape_name, lens, keep):
    # layer input, query and KV cache alone (X, Q, K, V): O, LSE, X2 and the MLP pre-activations G, U are
    # recomputed by the library -- on the kept rows only when a loss mask compacts the row-local part;
    # the oracle completes the same rounded four tensors in fp64
    from oracle import complete_record
    import paper_2503_01066_amd as A
    cu = synth.ragged_cu(lens)
    shp, osh, W, rec, dY = make_case(shape_name, dtype, cu, 23, "forward", wstd=0.3 if shape_name == "tiny" else 0.02,
                                     dy_std=1.0 if dtype == "f32" else 0.01)
    T = int(cu[-1])
    mask = None if keep is None else synth.keep_mask(T, keep, 5)
    Wd_ = {k: to_dev(v, dtype) for k, v in W.items()}
    for keys in (("X", "Q", "K", "V"), ("X", "Q", "K", "V", "U"), ("X", "X2", "Q", "K", "V", "O", "LSE", "G")):
        part = {k: rec[k] for k in keys}
        full = complete_record(osh, cu, {k: np.asarray(v, dtype=np.float64) for k, v in part.items()}, f64(W))
        ref = layer_backward_reuse(osh, cu, None, full, f64(W), dY, mask)
        d = {k: (torch.from_numpy(v).cuda() if k == "LSE" else to_dev(v, dtype)) for k, v in part.items()}
        out = A.alch_layer_backward(alch_shape(shp, dtype), A.Batch(cu), d, Wd_, to_dev(dY, dtype),
                                    loss_mask=None if mask is None else torch.from_numpy(mask).cuda())
        torch.cuda.synchronize()
        compare({k: to_np(v) for k, v in out.items()}, ref, dtype)


@pytest.mark.parametrize("keep", [0.0, 0.3, 1.0])
def test_loss_mask_row_compaction_bf16(keep):
    # bf16 with a loss mask runs the row-local part on the kept rows only (row count on the device);
    # the result must still be the dense backward with the masked dY rows zeroed (the oracle's definition),
    # including the degenerate masks "nothing kept" and "everything kept" and a ragged, multi-tile T
    cu = synth.ragged_cu([300, 1, 257, 64, 409])
    T = int(cu[-1])
    shp, osh, W, rec, dY = make_case("medium", "bf16", cu, 23, "drawn", dy_std=0.01)
    mask = synth.keep_mask(T, keep, 5)
    ref = layer_backward_reuse(osh, cu, None, f64(rec), f64(W), dY, mask)
    gpu = run_gpu(shp, "bf16", cu, W, rec, dY, loss_mask=mask)
    for k in gpu:
        assert np.isfinite(gpu[k]).all(), k
        if np.abs(ref[k]).max() == 0:
            assert np.abs(gpu[k]).max() == 0, k
        else:
            assert rel_err(gpu[k], ref[k]) <= TOL["bf16"], (k, rel_err(gpu[k], ref[k]))
