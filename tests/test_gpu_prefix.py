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
         ("f32", "tiny", [0, 3], [[2], [1, 1]]),            # an empty prompt: its response stands alone
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


@pytest.mark.parametrize("dtype,shape_name,prompts,responses", [CASES[0], CASES[3]])
def test_partial_record_with_shared_prefixes(dtype, shape_name, prompts, responses):
    # X, Q, K, V only: O and LSE are recomputed by the shared-prefix attention forward, then X2, G, U
    import paper_2503_01066_amd as A
    shp, osh, b, W, X, _, rec64, rec, dY = make(dtype, shape_name, prompts, responses, 21)
    four = {k: rec[k] for k in ("X", "Q", "K", "V")}
    # the oracle completes the same rounded tensors: attention over the visibility of the batch
    from oracle.prefix import _attention, visibility
    from oracle.layer import _rms_norm
    T = X.shape[0]
    Hq, Hkv, D = osh.n_q_heads, osh.n_kv_heads, osh.head_dim
    W64 = f64(W)
    Q, K, V = (np.asarray(four[k], dtype=np.float64) for k in ("Q", "K", "V"))
    O, LSE = _attention(osh, visibility(b["cu"], b["prefix"]), Q.reshape(T, Hq, D), K.reshape(T, Hkv, D), V.reshape(T, Hkv, D))
    full = dict(f64(four), O=O.reshape(T, Hq * D), LSE=LSE)
    full["X2"] = full["X"] + full["O"] @ W64["Wo"].T
    H2, _ = _rms_norm(full["X2"], W64["g2"], osh.rms_eps)
    full["G"], full["U"] = H2 @ W64["Wg"].T, H2 @ W64["Wu"].T
    ref = layer_backward_reuse_prefix(osh, b["cu"], b["prefix"], full, W64, dY)
    batch = A.Batch(b["cu"], positions=b["positions"], prefix=b["prefix"])
    out = A.alch_layer_backward(alch_shape(shp, dtype), batch, {k: to_dev(v, dtype) for k, v in four.items()},
                                {k: to_dev(v, dtype) for k, v in W.items()}, to_dev(dY, dtype))
    torch.cuda.synchronize()
    for k in ["dX"] + ["d" + w for w in WEIGHT_KEYS]:
        assert rel_err(to_np(out[k]), ref[k]) <= TOL[dtype], (k, rel_err(to_np(out[k]), ref[k]))


@pytest.mark.parametrize("dtype,shape_name,prompts,responses", [CASES[0], CASES[3]])
def test_loss_mask_on_a_shared_prefix_batch(dtype, shape_name, prompts, responses):
    # loss mask = zeroed dY rows (the prompt rows of a top layer carry no loss): the row-local part may run on the
    # kept rows only, the attention backward still reaches the prompt's keys and values
    import paper_2503_01066_amd as A
    shp, osh, b, W, X, _, _, rec, dY = make(dtype, shape_name, prompts, responses, 31)
    T = X.shape[0]
    mask = np.zeros(T, np.uint8)
    mask[int(b["cu"][b["n_prompts"]]):] = 1          # responses only
    mask[np.asarray(b["cu"][1:b["n_prompts"] + 1]) - 1] = 1   # and the last row of every prompt
    dYz = dY.copy()
    dYz[mask == 0] = 0
    ref = layer_backward_reuse_prefix(osh, b["cu"], b["prefix"], f64(rec), f64(W), dYz)
    batch = A.Batch(b["cu"], positions=b["positions"], prefix=b["prefix"])
    out = A.alch_layer_backward(alch_shape(shp, dtype), batch, dev_record(rec, dtype), {k: to_dev(v, dtype) for k, v in W.items()},
                                to_dev(dY, dtype), loss_mask=torch.from_numpy(mask).cuda())
    torch.cuda.synchronize()
    for k in ["dX"] + ["d" + w for w in WEIGHT_KEYS]:
        assert rel_err(to_np(out[k]), ref[k]) <= TOL[dtype], (k, rel_err(to_np(out[k]), ref[k]))


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


# ---- DPO head and the stack under it ------------------------------------------------------------
from oracle.prefix import stack_forward_prefix, stack_backward_dpo


def make_dpo_stack(dtype, shape_name, prompts, responses, L, V, seed):
    shp = synth.shape_dict(shape_name)
    osh = oracle_shape(shp)
    b = synth.preference_batch(prompts, responses, V, seed)
    T = int(b["cu"][-1])
    wstd = 0.3 if shape_name == "tiny" else 0.05
    Ws = [synth.layer_weights(shp, seed + 10 * l, dtype, std=wstd, gain_std=0.1) for l in range(L)]
    rng = np.random.default_rng(seed + 1000)
    X0 = synth.normal(rng, (T, shp["hidden"]), 1.0, dtype)
    gf = synth.quantize(1.0 + 0.1 * rng.standard_normal(shp["hidden"]).astype(np.float32), dtype)
    Wlm = synth.normal(rng, (V, shp["hidden"]), wstd, dtype)
    n_slots = sum(len(r) for r in responses)
    ref = rng.normal(-3.0, 1.0, n_slots).astype(np.float32)
    Xf64, recs64 = stack_forward_prefix(osh, b["cu"], b["prefix"], X0.astype(np.float64), [f64(W) for W in Ws])
    recs = []
    for r in recs64:
        q = {k: synth.quantize(r[k].astype(np.float32), dtype) for k in REC}
        q["LSE"] = r["LSE"].astype(np.float32)
        recs.append(q)
    Xf = synth.quantize(Xf64.astype(np.float32), dtype)
    return shp, osh, b, Ws, recs, Xf, gf, Wlm, ref


@pytest.mark.parametrize("dtype,shape_name,prompts,responses,V", [
    ("f32", "tiny", [4, 3], [[3, 2], [2, 5]], 53),
    ("bf16", "medium", [150, 70], [[60, 33], [129, 20]], 1024),
    ("bf16", "medium64", [90], [[40, 40]], 512)])
def test_stack_backward_dpo_matches_oracle(dtype, shape_name, prompts, responses, V):
    import paper_2503_01066_amd as A
    L, beta = 2, 0.5
    shp, osh, b, Ws, recs, Xf, gf, Wlm, ref = make_dpo_stack(dtype, shape_name, prompts, responses, L, V, 3)
    want = stack_backward_dpo(osh, b["cu"], b["prefix"], [f64(r) for r in recs], [f64(W) for W in Ws], Xf.astype(np.float64),
                              gf.astype(np.float64), Wlm.astype(np.float64), b["item_row"], b["item_label"], b["item_slot"],
                              ref.astype(np.float64), beta)
    batch = A.Batch(b["cu"], positions=b["positions"], prefix=b["prefix"])
    out = A.alch_stack_backward_dpo(alch_shape(shp, dtype), batch, [dev_record(r, dtype) for r in recs],
                                    [{k: to_dev(v, dtype) for k, v in W.items()} for W in Ws], to_dev(Xf, dtype),
                                    to_dev(gf, dtype), to_dev(Wlm, dtype), b["item_row"], b["item_label"], b["item_slot"],
                                    ref, beta)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    # z and the loss come from sums of log-probabilities over up to a hundred tokens: absolute bar on that scale
    zscale = max(1.0, np.abs(want["z"]).max())
    assert np.abs(to_np(out["z"]) - want["z"]).max() <= tol * zscale * 5, (to_np(out["z"]), want["z"])
    assert abs(out["loss"].item() - want["loss"]) <= tol * max(1.0, abs(want["loss"])) * 5
    for k in ("dX_embed", "dg_final", "dW_lm"):
        assert rel_err(to_np(out[k]), want[k]) <= tol * (3 if dtype == "bf16" else 1), (k, rel_err(to_np(out[k]), want[k]))
    for l in range(L):
        for k in WEIGHT_KEYS:
            e = rel_err(to_np(out["layers"][l]["d" + k]), want["layers"][l]["d" + k])
            assert e <= tol * (3 if dtype == "bf16" else 1), (l, k, e)


def test_dpo_without_pairs_gives_zero():
    import paper_2503_01066_amd as A
    dtype = "f32"
    shp, osh, b, Ws, recs, Xf, gf, Wlm, ref = make_dpo_stack(dtype, "tiny", [4], [[]], 1, 17, 1)
    batch = A.Batch(b["cu"], positions=b["positions"], prefix=b["prefix"])
    out = A.alch_stack_backward_dpo(alch_shape(shp, dtype), batch, [dev_record(r, dtype) for r in recs],
                                    [{k: to_dev(v, dtype) for k, v in W.items()} for W in Ws], to_dev(Xf, dtype),
                                    to_dev(gf, dtype), to_dev(Wlm, dtype), b["item_row"], b["item_label"], b["item_slot"],
                                    np.zeros(0, np.float32), 0.5)
    torch.cuda.synchronize()
    assert out["loss"].item() == 0.0
    for k in ("dX_embed", "dg_final", "dW_lm"):
        assert float(out[k].abs().max()) == 0.0, k


def test_stack_backward_dpo_with_adapters_on_a_frozen_base():
    # the paper's training setting (Section 6): rank-8 adapters, frozen base and head, DPO loss
    import paper_2503_01066_amd as A
    from oracle.lora import merged_weights
    from oracle.prefix import stack_backward_dpo_lora
    dtype, L, V, beta, rank, scale = "bf16", 2, 1024, 0.5, 8, 2.0
    shp = synth.shape_dict("medium")
    osh = oracle_shape(shp)
    b = synth.preference_batch([150, 70], [[60, 33], [129, 20]], V, 4)
    T = int(b["cu"][-1])
    Ws = [synth.layer_weights(shp, 4 + 10 * l, dtype, std=0.05, gain_std=0.1) for l in range(L)]
    loras = [synth.lora_adapters(shp, rank, 70 + l, dtype, projections=pj) for l, pj in
             enumerate((synth.PROJECTIONS, ("q", "v", "d")))]
    rng = np.random.default_rng(1004)
    X0 = synth.normal(rng, (T, shp["hidden"]), 1.0, dtype)
    gf = synth.quantize(1.0 + 0.1 * rng.standard_normal(shp["hidden"]).astype(np.float32), dtype)
    Wlm = synth.normal(rng, (V, shp["hidden"]), 0.05, dtype)
    ref = rng.normal(-3.0, 1.0, 4).astype(np.float32)
    merged = [merged_weights(f64(W), {p: (a.astype(np.float64), bb.astype(np.float64)) for p, (a, bb) in lo.items()}, scale)
              for W, lo in zip(Ws, loras)]
    Xf64, recs64 = stack_forward_prefix(osh, b["cu"], b["prefix"], X0.astype(np.float64), merged)
    recs = []
    for r in recs64:
        q = {k: synth.quantize(r[k].astype(np.float32), dtype) for k in REC}
        q["LSE"] = r["LSE"].astype(np.float32)
        recs.append(q)
    Xf = synth.quantize(Xf64.astype(np.float32), dtype)
    lo64 = [{p: (a.astype(np.float64), bb.astype(np.float64)) for p, (a, bb) in lo.items()} for lo in loras]
    want = stack_backward_dpo_lora(osh, b["cu"], b["prefix"], [f64(r) for r in recs], [f64(W) for W in Ws], lo64, scale,
                                   Xf.astype(np.float64), gf.astype(np.float64), Wlm.astype(np.float64), b["item_row"],
                                   b["item_label"], b["item_slot"], ref.astype(np.float64), beta)
    batch = A.Batch(b["cu"], positions=b["positions"], prefix=b["prefix"])
    dlo = [{p: (to_dev(a, dtype), to_dev(bb, dtype)) for p, (a, bb) in lo.items()} for lo in loras]
    out = A.alch_stack_backward_dpo(alch_shape(shp, dtype), batch, [dev_record(r, dtype) for r in recs],
                                    [{k: to_dev(v, dtype) for k, v in W.items()} for W in Ws], to_dev(Xf, dtype),
                                    to_dev(gf, dtype), to_dev(Wlm, dtype), b["item_row"], b["item_label"], b["item_slot"],
                                    ref, beta, lora_layers=dlo, rank=rank, scale=scale, want=(), want_head=False)
    torch.cuda.synchronize()
    tol = TOL[dtype] * 3
    assert abs(out["loss"].item() - want["loss"]) <= tol * max(1.0, abs(want["loss"]))
    assert out["dW_lm"] is None and out["dg_final"] is None
    assert rel_err(to_np(out["dX_embed"]), want["dX_embed"]) <= tol
    for l, lo in enumerate(loras):
        assert not any(k.startswith("dW") for k in out["layers"][l])
        for p in lo:
            for k in ("dA" + p, "dB" + p):
                e = rel_err(to_np(out["layers"][l][k]), want["layers"][l][k])
                assert e <= tol, (l, k, e)


@pytest.mark.parametrize("seed", range(4))
def test_layer_backward_random_prefix_batches(seed):
    # seeded random batches: 1-3 prompts of 1-400 tokens, 0-3 responses of 0-200 tokens each, on the matrix-core path
    import paper_2503_01066_amd as A
    rng = np.random.default_rng(100 + seed)
    n_p = int(rng.integers(1, 4))
    prompts = [int(rng.integers(1, 401)) for _ in range(n_p)]
    responses = [[int(rng.integers(0, 201)) for _ in range(int(rng.integers(0, 4)))] for _ in range(n_p)]
    dtype = "bf16"
    shp, osh, b, W, X, _, _, rec, dY = make(dtype, "medium", prompts, responses, 40 + seed)
    ref = layer_backward_reuse_prefix(osh, b["cu"], b["prefix"], f64(rec), f64(W), dY)
    batch = A.Batch(b["cu"], positions=b["positions"], prefix=b["prefix"])
    out = A.alch_layer_backward(alch_shape(shp, dtype), batch, dev_record(rec, dtype),
                                {k: to_dev(v, dtype) for k, v in W.items()}, to_dev(dY, dtype))
    torch.cuda.synchronize()
    for k in ["dX"] + ["d" + w for w in WEIGHT_KEYS]:
        assert rel_err(to_np(out[k]), ref[k]) <= TOL[dtype], (prompts, responses, k, rel_err(to_np(out[k]), ref[k]))


@pytest.mark.parametrize("dtype,shape_name,V", [("f32", "tiny", 61), ("bf16", "medium", 1024), ("bf16", "medium", 1001),
                                                ("bf16", "medium", 20032)])
def test_dpo_head_alone_with_more_items_than_one_chunk(dtype, shape_name, V):
    # no layers: the call is the DPO head + final-norm backward.  9,000 scored tokens exceed the 8,192-row chunk of
    # the head, so the logits of every chunk are formed twice (log-probabilities, then gradients); rows score
    # zero, one or two tokens
    import paper_2503_01066_amd as A
    from oracle.prefix import dpo_head
    shp = synth.shape_dict(shape_name)
    osh = oracle_shape(shp)
    H, T, M, n_pairs = shp["hidden"], 9500, 9000, 3
    rng = np.random.default_rng(12)
    Xf = synth.normal(rng, (T, H), 1.0, dtype)
    gf = synth.quantize(1.0 + 0.1 * rng.standard_normal(H).astype(np.float32), dtype)
    Wlm = synth.normal(rng, (V, H), 0.3 if shape_name == "tiny" else 0.05, dtype)
    rows = np.sort(rng.integers(0, T, M)).astype(np.int32)
    labels = rng.integers(0, V, M).astype(np.int32)
    slots = rng.integers(0, 2 * n_pairs, M).astype(np.int32)
    # per-token log-probabilities are about -log V: a reference near the policy keeps z of order one
    ref = np.array([-(slots == s).sum() * np.log(V) for s in range(2 * n_pairs)], np.float32) + rng.normal(0, 1, 2 * n_pairs).astype(np.float32)
    beta = 0.05
    loss, dX, dg, dW, z = dpo_head(osh, Xf.astype(np.float64), gf.astype(np.float64), Wlm.astype(np.float64), rows, labels, slots,
                                   ref.astype(np.float64), beta)
    cu = synth.ragged_cu([T])
    out = A.alch_stack_backward_dpo(alch_shape(shp, dtype), A.Batch(cu), [], [], to_dev(Xf, dtype), to_dev(gf, dtype),
                                    to_dev(Wlm, dtype), rows, labels, slots, ref, beta)
    torch.cuda.synchronize()
    _check_dpo_head(out, loss, dX, dg, dW, z, TOL[dtype], "dpo head %s V=%d" % (dtype, V))


def _check_dpo_head(out, loss, dX, dg, dW, z, tol, label):
    zs = max(1.0, np.abs(z).max())
    ez = np.abs(to_np(out["z"]) - z).max() / zs
    el = abs(out["loss"].item() - loss) / max(1.0, abs(loss))
    errs = {k: rel_err(to_np(out[k]), want) for k, want in (("dX_embed", dX), ("dg_final", dg), ("dW_lm", dW))}
    print(label, "z %.3e loss %.3e" % (ez, el), {k: "%.3e" % e for k, e in errs.items()}, flush=True)
    assert ez <= tol and el <= tol, (label, ez, el)
    for k, e in errs.items():
        assert e <= tol, (label, k, e)


def test_dpo_head_alone_at_the_real_vocabulary():
    # vocabulary 128,256, hidden 4096: every thread of the one-row-in-registers log-probability kernel holds 15 or 16
    # eight-logit chunks; labels anywhere in the vocabulary; rows that score zero, one or two tokens
    import paper_2503_01066_amd as A
    from oracle.prefix import dpo_head
    dtype, V = "bf16", 128256
    shp = synth.shape_dict("llama8b")
    osh = oracle_shape(shp)
    H, T, M, n_pairs = shp["hidden"], 2300, 2000, 4
    rng = np.random.default_rng(31)
    Xf = synth.normal(rng, (T, H), 1.0, dtype)
    gf = synth.quantize(1.0 + 0.1 * rng.standard_normal(H).astype(np.float32), dtype)
    Wlm = synth.normal(rng, (V, H), 0.02, dtype)
    rows = np.sort(rng.integers(0, T, M)).astype(np.int32)
    labels = rng.integers(0, V, M).astype(np.int32)
    slots = rng.integers(0, 2 * n_pairs, M).astype(np.int32)
    ref = np.array([-(slots == s).sum() * np.log(V) for s in range(2 * n_pairs)], np.float32) + rng.normal(0, 1, 2 * n_pairs).astype(np.float32)
    beta = 0.05
    out = A.alch_stack_backward_dpo(alch_shape(shp, dtype), A.Batch(synth.ragged_cu([T])), [], [], to_dev(Xf, dtype),
                                    to_dev(gf, dtype), to_dev(Wlm, dtype), rows, labels, slots, ref, beta)
    torch.cuda.synchronize()
    out = {k: (v.float().cpu() if torch.is_tensor(v) else v) for k, v in out.items()}
    torch.cuda.empty_cache()
    loss, dX, dg, dW, z = dpo_head(osh, Xf.astype(np.float64), gf.astype(np.float64), Wlm.astype(np.float64), rows, labels, slots,
                                   ref.astype(np.float64), beta)
    _check_dpo_head(out, loss, dX, dg, dW, z, TOL[dtype], "dpo head V=128256")
