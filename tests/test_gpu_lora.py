"""GPU parity of alch_layer_backward_lora (Section 3 assumption A1, Section 6: rank-8 adapters on a
frozen base) against the fp64 oracle on the same seeded inputs.
Bar: per output tensor max|gpu - oracle| / max|oracle| <= 2e-2 (bf16) / 1e-4 (f32)."""
import numpy as np
import pytest
import torch

import synth_inputs as synth
from helpers import TOL, to_dev, to_np, f64, rel_err, cosine, oracle_shape, alch_shape
from oracle import attention_lse, WEIGHT_KEYS
from oracle.lora import layer_forward_lora, layer_backward_reuse_lora

pytestmark = pytest.mark.gpu
REC = ("X", "X2", "Q", "K", "V", "O", "G", "U")


def make_case(shape_name, dtype, cu, seed, rank, projections, record="forward", wstd=0.02, dy_std=1.0, scale=2.0,
              lora_std=0.05):
    shp = synth.shape_dict(shape_name)
    osh = oracle_shape(shp)
    T = int(cu[-1])
    W = synth.layer_weights(shp, seed, dtype, std=wstd, gain_std=0.1)
    lora = synth.lora_adapters(shp, rank, seed + 7, dtype, projections, std=lora_std)
    lora64 = {p: (a.astype(np.float64), b.astype(np.float64)) for p, (a, b) in lora.items()}
    if record == "forward":
        X = synth.activations(T, shp["hidden"], seed + 1, dtype)
        _, rec64 = layer_forward_lora(osh, cu, None, X.astype(np.float64), f64(W), lora64, scale)
        rec = {k: synth.quantize(rec64[k].astype(np.float32), dtype) for k in REC}
        rec["LSE"] = rec64["LSE"].astype(np.float32)
    else:
        rec = synth.drawn_record(shp, T, seed + 1, dtype)
        rec["LSE"] = attention_lse(osh, cu, rec["Q"].astype(np.float64), rec["K"].astype(np.float64)).astype(np.float32)
    dY = synth.activations(T, shp["hidden"], seed + 2, dtype, std=dy_std)
    return shp, osh, W, lora, lora64, rec, dY, scale


def run_gpu(shp, dtype, cu, W, lora, rank, scale, rec, dY, loss_mask=None, want=(), **kw):
    import paper_2503_01066_amd as A
    batch = A.Batch(cu)
    dW = {k: to_dev(v, dtype) for k, v in W.items()}
    dl = {p: (to_dev(a, dtype), to_dev(b, dtype)) for p, (a, b) in lora.items()}
    drec = {k: to_dev(rec[k], dtype) for k in REC}
    drec["LSE"] = torch.from_numpy(rec["LSE"]).cuda()
    dm = None if loss_mask is None else torch.from_numpy(loss_mask).cuda()
    out = A.alch_layer_backward_lora(alch_shape(shp, dtype), batch, drec, dW, dl, rank, scale, to_dev(dY, dtype),
                                     loss_mask=dm, want=want, **kw)
    torch.cuda.synchronize()
    return {k: to_np(v) for k, v in out.items()}


def compare(gpu, ref, dtype):
    for k in gpu:
        e = rel_err(gpu[k], ref[k])
        assert np.isfinite(gpu[k]).all(), k
        assert e <= TOL[dtype], (k, e, cosine(gpu[k], ref[k]))


def test_config1_fp32_all_adapters_with_loss_mask():
    cu = synth.uniform_cu(2, 128)
    shp, osh, W, lora, lora64, rec, dY, scale = make_case("config1", "f32", cu, 0, 8, synth.PROJECTIONS)
    mask = synth.keep_mask(256, 0.5, 0)
    for lm in (None, mask):
        ref = layer_backward_reuse_lora(osh, cu, None, f64(rec), f64(W), lora64, scale, dY, lm)
        gpu = run_gpu(shp, "f32", cu, W, lora, 8, scale, rec, dY, loss_mask=lm, want=WEIGHT_KEYS)
        assert sorted(gpu) == sorted(ref)
        compare(gpu, ref, "f32")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_tiny_ragged_frozen_base_q_v_only(dtype):
    # the usual adapter placement (query and value projections), frozen base, empty and 1-token sequences
    cu = synth.ragged_cu([1, 5, 0, 8, 3])
    shp, osh, W, lora, lora64, rec, dY, scale = make_case("tiny", dtype, cu, 3, 8, ("q", "v"), wstd=0.3, lora_std=0.2)
    ref = layer_backward_reuse_lora(osh, cu, None, f64(rec), f64(W), lora64, scale, dY)
    gpu = run_gpu(shp, dtype, cu, W, lora, 8, scale, rec, dY)
    assert sorted(gpu) == ["dAq", "dAv", "dBq", "dBv", "dX"]
    compare(gpu, ref, dtype)


@pytest.mark.parametrize("shape_name,lens,rank,projections", [
    ("medium", [300, 1, 257, 64], 8, synth.PROJECTIONS),
    ("medium64", [130, 200, 77], 16, ("q", "k", "o", "u")),
    ("medium", [715, 128, 33], 64, ("v", "g", "d")),
])
def test_medium_bf16_ranks_and_subsets(shape_name, lens, rank, projections):
    cu = synth.ragged_cu(lens)
    for record in ("drawn", "forward"):
        shp, osh, W, lora, lora64, rec, dY, scale = make_case(shape_name, "bf16", cu, 5, rank, projections, record,
                                                               dy_std=0.01, scale=16.0 / rank)
        ref = layer_backward_reuse_lora(osh, cu, None, f64(rec), f64(W), lora64, scale, dY)
        gpu = run_gpu(shp, "bf16", cu, W, lora, rank, scale, rec, dY, want=WEIGHT_KEYS)
        compare(gpu, ref, "bf16")


def test_accumulate_adds_to_adapter_gradients():
    import paper_2503_01066_amd as A
    cu = synth.ragged_cu([200, 56])
    shp, osh, W, lora, lora64, rec, dY, scale = make_case("medium64", "bf16", cu, 9, 8, ("q", "d"), "drawn", dy_std=0.01)
    ref = layer_backward_reuse_lora(osh, cu, None, f64(rec), f64(W), lora64, scale, dY)
    rng = np.random.default_rng(1)
    init = {}
    for p, (a, b) in lora.items():
        init["dA" + p] = synth.quantize(rng.standard_normal(a.shape).astype(np.float32) * np.abs(ref["dA" + p]).max(), "bf16")
        init["dB" + p] = synth.quantize(rng.standard_normal(b.shape).astype(np.float32) * np.abs(ref["dB" + p]).max(), "bf16")
    bufs = {k: to_dev(v, "bf16") for k, v in init.items()}
    gpu = run_gpu(shp, "bf16", cu, W, lora, 8, scale, rec, dY, lora_grads=bufs, accumulate=True)
    for k in init:
        assert rel_err(gpu[k], ref[k] + init[k]) <= TOL["bf16"], k


def test_adapters_absent_equals_plain_backward():
    # every adapter NULL: the call must give what alch_layer_backward gives, bit for bit
    import paper_2503_01066_amd as A
    cu = synth.ragged_cu([100, 156])
    shp, osh, W, lora, lora64, rec, dY, scale = make_case("medium", "bf16", cu, 11, 8, (), "drawn", dy_std=0.01)
    a = run_gpu(shp, "bf16", cu, W, {}, 8, 1.0, rec, dY, want=WEIGHT_KEYS)
    batch = A.Batch(cu)
    drec = {k: to_dev(rec[k], "bf16") for k in REC}
    drec["LSE"] = torch.from_numpy(rec["LSE"]).cuda()
    b = A.alch_layer_backward(alch_shape(shp, "bf16"), batch, drec, {k: to_dev(v, "bf16") for k, v in W.items()},
                              to_dev(dY, "bf16"))
    torch.cuda.synchronize()
    for k in a:
        assert np.array_equal(a[k], to_np(b[k])), k


def test_llama8b_width_frozen_base_short_batch():
    # the paper's setting at real layer width: frozen 8B-shaped base, rank 8 on all projections, T = 320
    cu = synth.ragged_cu([190, 130])
    shp, osh, W, lora, lora64, rec, dY, scale = make_case("llama8b", "bf16", cu, 13, 8, synth.PROJECTIONS, "drawn",
                                                           dy_std=0.01, scale=2.0)
    ref = layer_backward_reuse_lora(osh, cu, None, f64(rec), f64(W), lora64, scale, dY)
    gpu = run_gpu(shp, "bf16", cu, W, lora, 8, scale, rec, dY)
    compare(gpu, ref, "bf16")


@pytest.mark.parametrize("dtype,shape_name,lens,L,V,wstd", [("f32", "tiny", [5, 1, 9], 3, 37, 0.3),
                                                           ("bf16", "medium64", [130, 61, 200], 2, 1000, 0.05)])
def test_stack_frozen_base_adapter_gradients(dtype, shape_name, lens, L, V, wstd):
    # the paper's training setting end to end: head + L adapted layers, frozen base and head, adapters on q and v
    # (layer 0) or on every projection (other layers); records from the adapted oracle forward
    import paper_2503_01066_amd as A
    from oracle.lora import stack_forward_lora, stack_backward_reuse_lora
    cu = synth.ragged_cu(lens)
    shp = synth.shape_dict(shape_name)
    osh = oracle_shape(shp)
    T = int(cu[-1])
    scale, rank = 2.0, 8
    Ws = [synth.layer_weights(shp, 40 + 10 * l, dtype, std=wstd, gain_std=0.1) for l in range(L)]
    loras = [synth.lora_adapters(shp, rank, 90 + l, dtype, ("q", "v") if l == 0 else synth.PROJECTIONS, std=0.1) for l in range(L)]
    loras64 = [{p: (a.astype(np.float64), b.astype(np.float64)) for p, (a, b) in lo.items()} for lo in loras]
    rng = np.random.default_rng(77)
    X0 = synth.normal(rng, (T, shp["hidden"]), 1.0, dtype)
    gf = synth.quantize(1.0 + 0.1 * rng.standard_normal(shp["hidden"]).astype(np.float32), dtype)
    Wlm = synth.normal(rng, (V, shp["hidden"]), wstd, dtype)
    ids = rng.integers(0, V, T)
    labels = np.full(T, -1, dtype=np.int32)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if b - a > 1:
            labels[a:b - 1] = ids[a + 1:b]
    Xf64, recs64 = stack_forward_lora(osh, cu, None, X0.astype(np.float64), [f64(W) for W in Ws], loras64, scale)
    recs = []
    for r in recs64:
        q = {k: synth.quantize(r[k].astype(np.float32), dtype) for k in REC}
        q["LSE"] = r["LSE"].astype(np.float32)
        recs.append(q)
    Xf = synth.quantize(Xf64.astype(np.float32), dtype)
    ref = stack_backward_reuse_lora(osh, cu, None, [f64(r) for r in recs], [f64(W) for W in Ws], loras64, scale,
                                    Xf.astype(np.float64), gf.astype(np.float64), Wlm.astype(np.float64), labels)

    drecs = []
    for r in recs:
        d = {k: to_dev(r[k], dtype) for k in REC}
        d["LSE"] = torch.from_numpy(r["LSE"]).cuda()
        drecs.append(d)
    out = A.alch_stack_backward_lora(alch_shape(shp, dtype), A.Batch(cu), drecs,
                                     [{k: to_dev(v, dtype) for k, v in W.items()} for W in Ws],
                                     [{p: (to_dev(a, dtype), to_dev(b, dtype)) for p, (a, b) in lo.items()} for lo in loras],
                                     rank, scale, to_dev(Xf, dtype), to_dev(gf, dtype), to_dev(Wlm, dtype),
                                     torch.from_numpy(labels).cuda())
    torch.cuda.synchronize()
    tol = TOL[dtype]
    assert abs(out["loss"].item() - ref["loss"]) <= tol * max(1.0, abs(ref["loss"]))
    assert rel_err(to_np(out["dX_embed"]), ref["dX_embed"]) <= tol
    assert out["dW_lm"] is None and out["dg_final"] is None
    for l in range(L):
        keys = sorted(out["layers"][l])
        assert keys == sorted("d" + m + p for p in loras[l] for m in "AB"), keys
        for k in keys:
            e = rel_err(to_np(out["layers"][l][k]), ref["layers"][l][k])
            assert e <= tol, (l, k, e)
