"""GPU parity of alch_stack_backward (cross-entropy head + layer walk) and alch_layer_forward
against the fp64 oracle."""
import numpy as np
import pytest
import torch

import synth_inputs as synth
from helpers import TOL, to_dev, to_np, f64, rel_err, oracle_shape, alch_shape, check_all
from oracle import stack_forward, stack_backward_reuse, layer_forward, layer_backward_recompute, WEIGHT_KEYS

pytestmark = pytest.mark.gpu
REC = ("X", "X2", "Q", "K", "V", "O", "G", "U")


def make_stack(shape_name, dtype, cu, L, V, seed, wstd):
    shp = synth.shape_dict(shape_name)
    osh = oracle_shape(shp)
    T = int(cu[-1])
    Ws = [synth.layer_weights(shp, seed + 10 * l, dtype, std=wstd, gain_std=0.1) for l in range(L)]
    rng = np.random.default_rng(seed + 1000)
    X0 = synth.normal(rng, (T, shp["hidden"]), 1.0, dtype)
    gf = synth.quantize(1.0 + 0.1 * rng.standard_normal(shp["hidden"]).astype(np.float32), dtype)
    Wlm = synth.normal(rng, (V, shp["hidden"]), wstd, dtype)
    ids = rng.integers(0, V, T)
    labels = np.full(T, -1, dtype=np.int32)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if b - a > 1:
            labels[a:b - 1] = ids[a + 1:b]
    # records: oracle forward in fp64, then rounded to the storage type (what a serving pass would hold)
    Xf64, recs64 = stack_forward(osh, cu, None, X0.astype(np.float64), [f64(W) for W in Ws])
    recs = []
    for r in recs64:
        q = {k: synth.quantize(r[k].astype(np.float32), dtype) for k in REC}
        q["LSE"] = r["LSE"].astype(np.float32)
        recs.append(q)
    Xf = synth.quantize(Xf64.astype(np.float32), dtype)
    return shp, osh, Ws, recs, Xf, gf, Wlm, labels


def run_stack(shp, dtype, cu, Ws, recs, Xf, gf, Wlm, labels, mask=None, hooks=None):
    import paper_2503_01066_amd as A
    batch = A.Batch(cu)
    dWs = [{k: to_dev(v, dtype) for k, v in W.items()} for W in Ws]
    drecs = []
    for r in recs:
        d = {k: to_dev(r[k], dtype) for k in REC if k in r}
        if "LSE" in r:
            d["LSE"] = torch.from_numpy(r["LSE"]).cuda()
        drecs.append(d)
    out = A.alch_stack_backward(alch_shape(shp, dtype), batch, drecs, dWs, to_dev(Xf, dtype), to_dev(gf, dtype),
                                to_dev(Wlm, dtype), torch.from_numpy(labels).cuda(),
                                loss_mask=None if mask is None else torch.from_numpy(mask).cuda(), hooks=hooks)
    torch.cuda.synchronize()
    return out


def check_stack(out, ref, dtype, L):
    tol = TOL[dtype]
    assert abs(out["loss"].item() - ref["loss"]) <= tol * max(1.0, abs(ref["loss"]))
    for k in ("dX_embed", "dg_final", "dW_lm"):
        assert rel_err(to_np(out[k]), ref[k]) <= tol, k
    for l in range(L):
        for k in WEIGHT_KEYS:
            assert rel_err(to_np(out["layers"][l]["d" + k]), ref["layers"][l]["d" + k]) <= tol, (l, k)


@pytest.mark.parametrize("dtype,shape_name,lens,V,wstd", [("f32", "tiny", [5, 1, 8], 53, 0.3),
                                                           ("bf16", "medium", [200, 150], 1024, 0.05)])
def test_stack_backward_matches_oracle(dtype, shape_name, lens, V, wstd):
    cu = synth.ragged_cu(lens)
    L = 2
    shp, osh, Ws, recs, Xf, gf, Wlm, labels = make_stack(shape_name, dtype, cu, L, V, 3, wstd)
    T = int(cu[-1])
    mask = np.ones(T, np.uint8)
    mask[::7] = 0
    for m in (None, mask):
        ref = stack_backward_reuse(osh, cu, None, [f64(r) for r in recs], [f64(W) for W in Ws], Xf.astype(np.float64),
                                   gf.astype(np.float64), Wlm.astype(np.float64), labels, m)
        out = run_stack(shp, dtype, cu, Ws, recs, Xf, gf, Wlm, labels, m)
        check_stack(out, ref, dtype, L)


def test_stack_nothing_counted_and_hooks():
    import paper_2503_01066_amd as A
    cu = synth.ragged_cu([6, 3])
    shp, osh, Ws, recs, Xf, gf, Wlm, labels = make_stack("tiny", "f32", cu, 3, 31, 5, 0.3)
    out = run_stack(shp, "f32", cu, Ws, recs, Xf, gf, Wlm, np.full(9, -1, np.int32))
    assert out["loss"].item() == 0.0
    assert float(out["dX_embed"].abs().max()) == 0.0 and float(out["dW_lm"].abs().max()) == 0.0
    # layers are walked output -> input; the preempt hook stops the walk
    seen = []
    out = run_stack(shp, "f32", cu, Ws, recs, Xf, gf, Wlm, labels, hooks=(lambda u, l: seen.append(l) or 0, None))
    assert seen == [2, 1, 0]
    with pytest.raises(A.AlchError) as e:
        run_stack(shp, "f32", cu, Ws, recs, Xf, gf, Wlm, labels, hooks=(None, lambda u, l: 1 if l == 1 else 0))
    assert e.value.code == -7
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype,shape_name,lens,wstd", [("f32", "config1", [128, 128], 0.02),
                                                         ("bf16", "medium", [300, 77, 1], 0.02),
                                                         ("bf16", "medium64", [90, 60], 0.05),
                                                         ("bf16", "odd", [33, 8], 0.3),
                                                         ("f32", "odd", [33, 8], 0.3)])
def test_layer_forward_and_reuse_equals_recompute(dtype, shape_name, lens, wstd):
    import paper_2503_01066_amd as A
    cu = synth.ragged_cu(lens)
    T = int(cu[-1])
    shp = synth.shape_dict(shape_name)
    osh = oracle_shape(shp)
    W = synth.layer_weights(shp, 11, dtype, std=wstd, gain_std=0.1)
    X = synth.activations(T, shp["hidden"], 12, dtype)
    dY = synth.activations(T, shp["hidden"], 13, dtype, std=0.5)
    Yref, rec_ref = layer_forward(osh, cu, None, X.astype(np.float64), f64(W))
    batch = A.Batch(cu)
    shape = alch_shape(shp, dtype)
    dW = {k: to_dev(v, dtype) for k, v in W.items()}
    Y, rec = A.alch_layer_forward(shape, batch, to_dev(X, dtype), dW)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    assert rel_err(to_np(Y), Yref) <= tol
    for k in REC + ("LSE",):
        assert rel_err(to_np(rec[k]), rec_ref[k]) <= tol, k
    # the paper's central claim on the device: gradients from the record the forward just produced
    # equal the gradients of a recomputed forward (oracle) under unchanged weights
    ref = layer_backward_recompute(osh, cu, None, X.astype(np.float64), f64(W), dY.astype(np.float64))
    out = A.alch_layer_backward(shape, batch, rec, dW, to_dev(dY, dtype))
    torch.cuda.synchronize()
    for k, v in out.items():
        assert rel_err(to_np(v), ref[k]) <= tol, (k, rel_err(to_np(v), ref[k]))


def test_stack_from_four_stream_records():
    # every layer's record holds X, Q, K, V only (Section 4.3.2: the rest is recomputed rather than kept);
    # the oracle completes the same rounded tensors in fp64 and walks the stack on them
    from oracle import complete_record
    cu = synth.ragged_cu([200, 150, 31])
    L, dtype = 3, "bf16"
    shp, osh, Ws, recs, Xf, gf, Wlm, labels = make_stack("medium", dtype, cu, L, 1024, 9, 0.05)
    T = int(cu[-1])
    four = [{k: r[k] for k in ("X", "Q", "K", "V")} for r in recs]
    full = [complete_record(osh, cu, f64(r), f64(W)) for r, W in zip(four, Ws)]
    for m in (None, synth.keep_mask(T, 0.4, 3)):
        ref = stack_backward_reuse(osh, cu, None, full, [f64(W) for W in Ws], Xf.astype(np.float64),
                                   gf.astype(np.float64), Wlm.astype(np.float64), labels, m)
        out = run_stack(shp, dtype, cu, Ws, four, Xf, gf, Wlm, labels, m)
        check_stack(out, ref, dtype, L)


@pytest.mark.parametrize("keep", [0.0, 0.3])
def test_stack_loss_mask_compacts_head_and_top_layer(keep):
    # bf16 with a loss mask: only counted tokens go through the LM head (two row chunks here: T > 8192) and the top
    # layer runs its row-local part on them; the result must equal the oracle's dense definition
    cu = synth.ragged_cu([3000, 2500, 3500])
    L, V = 1, 1024
    shp, osh, Ws, recs, Xf, gf, Wlm, labels = make_stack("medium", "bf16", cu, L, V, 11, 0.05)
    T = int(cu[-1])
    mask = synth.keep_mask(T, keep, 2)
    ref = stack_backward_reuse(osh, cu, None, [f64(r) for r in recs], [f64(W) for W in Ws], Xf.astype(np.float64),
                               gf.astype(np.float64), Wlm.astype(np.float64), labels, mask)
    out = run_stack(shp, "bf16", cu, Ws, recs, Xf, gf, Wlm, labels, mask)
    if keep == 0.0:
        assert out["loss"].item() == 0.0
        for k in ("dX_embed", "dg_final", "dW_lm"):
            assert float(out[k].abs().max()) == 0.0, k
    else:
        check_stack(out, ref, "bf16", L)


def _head_case(shape_name, V, lens, seed, dtype="bf16", wstd=0.02):
    """Inputs of the head alone (no layers): saved stack output, final gain, LM head, next-token labels drawn
    uniformly over the whole vocabulary (the last position of every sequence is ignored)."""
    shp = synth.shape_dict(shape_name)
    cu = synth.ragged_cu(lens)
    T, H = int(cu[-1]), shp["hidden"]
    rng = np.random.default_rng(seed)
    Xf = synth.normal(rng, (T, H), 1.0, dtype)
    gf = synth.quantize(1.0 + 0.1 * rng.standard_normal(H).astype(np.float32), dtype)
    Wlm = synth.normal(rng, (V, H), wstd, dtype)
    labels = rng.integers(0, V, T).astype(np.int32)
    labels[np.asarray(cu[1:]) - 1] = -1
    return shp, cu, Xf, gf, Wlm, labels


def _check_head(shp, cu, Xf, gf, Wlm, labels, mask, label, oracle_labels=None):
    from oracle.stack import _head_loss_and_grads
    out = run_stack(shp, "bf16", cu, [], [], Xf, gf, Wlm, labels, mask)
    out = {k: (v.float().cpu() if torch.is_tensor(v) else v) for k, v in out.items()}
    torch.cuda.empty_cache()
    loss, dX, dg, dW = _head_loss_and_grads(oracle_shape(shp), Xf.astype(np.float64), gf.astype(np.float64),
                                            Wlm.astype(np.float64), labels if oracle_labels is None else oracle_labels, mask)
    print("%s loss gpu %.6f oracle %.6f" % (label, out["loss"].item(), loss), flush=True)
    assert abs(out["loss"].item() - loss) <= 2e-2 * max(1.0, abs(loss))
    check_all(out, dict(dX_embed=dX, dg_final=dg, dW_lm=dW), 2e-2, label, keys=("dX_embed", "dg_final", "dW_lm"))


@pytest.mark.parametrize("keep", [None, 0.5])
def test_head_alone_at_the_real_vocabulary(keep):
    # the head config 4 runs: vocabulary 128,256 (16,032 eight-logit chunks per row, so every thread of the
    # one-row-in-registers cross-entropy kernel holds 15 or 16 chunks and the label falls in any of them), hidden
    # 4096, ragged rows; with a loss mask the counted rows are compacted first
    shp, cu, Xf, gf, Wlm, labels = _head_case("llama8b", 128256, [1200, 1, 900, 499], 21)
    mask = None if keep is None else synth.keep_mask(int(cu[-1]), keep, 22)
    _check_head(shp, cu, Xf, gf, Wlm, labels, mask, "head V=128256 keep=%s" % keep)


@pytest.mark.parametrize("keep", [None, 0.9])
def test_head_alone_second_row_chunk_and_labels_beyond_the_vocabulary(keep):
    # 8,300 dense rows: the second 8,192-row chunk of the head is not empty (labels, row losses and the accumulation
    # of dW_lm across chunks at a row offset); 20,032 logits per row = three register chunks per thread.  Labels at or
    # beyond the vocabulary are ignored positions, like negative ones.
    shp, cu, Xf, gf, Wlm, labels = _head_case("medium", 20032, [5000, 3300], 23, wstd=0.05)
    T = int(cu[-1])
    beyond = np.random.default_rng(5).choice(T, 40, replace=False)
    labels[beyond] = 20032 + (beyond % 7)
    oracle_labels = labels.copy()
    oracle_labels[beyond] = -1
    mask = None if keep is None else synth.keep_mask(T, keep, 24)
    _check_head(shp, cu, Xf, gf, Wlm, labels, mask, "head V=20032 T=8300 keep=%s" % keep, oracle_labels)
