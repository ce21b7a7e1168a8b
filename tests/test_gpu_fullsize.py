"""Full-size parity in the launch configurations bench.py times: config 2 (one Llama-3-8B-shaped layer,
bf16, 4 x 2048 tokens) and config 5 (one Llama-3-70B-shaped layer, 2 x 4096 tokens, dense and with the
loss mask), every output element by element against the fp64 oracle; full-width / short-batch cases;
config-3-sized capture/pack; the adapter mode at config-2 size on sampled outputs."""
import numpy as np
import pytest
import torch

import synth_inputs as synth
from helpers import to_dev, to_np, f64, rel_err, oracle_shape, alch_shape, check_all
from oracle import layer_backward_reuse, attention_lse, gather_pack, WEIGHT_KEYS

pytestmark = pytest.mark.gpu
REC = ("X", "X2", "Q", "K", "V", "O", "G", "U")


def gpu_layer(shp, cu, W, rec, dY):
    import paper_2503_01066_amd as A
    dW = {k: to_dev(v, "bf16") for k, v in W.items()}
    drec = {k: to_dev(rec[k], "bf16") for k in REC}
    drec["LSE"] = torch.from_numpy(rec["LSE"]).cuda()
    out = A.alch_layer_backward(alch_shape(shp, "bf16"), A.Batch(cu), drec, dW, to_dev(dY, "bf16"))
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("shape_name", ["llama8b", "phi4"])
def test_real_layer_width_short_batch_elementwise(shape_name):
    # every GEMM dimension at its real width (Llama-3-8B / Mistral-7B: hidden 4096, ffn 14336, 32/8 heads x 128;
    # Phi-4: hidden 5120, ffn 17920, 40/10 heads x 128 -- tile counts that are not powers of two), ragged short batch
    shp = synth.shape_dict(shape_name)
    osh = oracle_shape(shp)
    cu = synth.ragged_cu([150, 41, 129])
    T = int(cu[-1])
    W = synth.layer_weights(shp, 0, "bf16")
    rec = synth.drawn_record(shp, T, 1, "bf16")
    rec["LSE"] = attention_lse(osh, cu, rec["Q"].astype(np.float64), rec["K"].astype(np.float64)).astype(np.float32)
    dY = synth.activations(T, shp["hidden"], 2, "bf16", std=0.01)
    print("oracle ...", flush=True)
    ref = layer_backward_reuse(osh, cu, None, f64(rec), f64(W), dY.astype(np.float64))
    print("gpu ...", flush=True)
    out = gpu_layer(shp, cu, W, rec, dY)
    for k, v in out.items():
        e = rel_err(to_np(v), ref[k])
        assert e <= 2e-2, (k, e)


def _full_size_layer(shape_name, B, S, mask_rate=None):
    """One bench-sized layer step (drawn record, LSE from the drawn Q, K), oracle and GPU on the same bits,
    every output compared element by element."""
    import paper_2503_01066_amd as A
    shp = synth.shape_dict(shape_name)
    osh = oracle_shape(shp)
    cu = synth.uniform_cu(B, S)
    T = B * S
    W = synth.layer_weights(shp, 0, "bf16")
    rec = synth.drawn_record(shp, T, 1, "bf16")
    print("lse ...", flush=True)
    rec["LSE"] = attention_lse(osh, cu, rec["Q"].astype(np.float64), rec["K"].astype(np.float64)).astype(np.float32)
    dY = synth.activations(T, shp["hidden"], 2, "bf16", std=0.01)
    mask = None if mask_rate is None else synth.keep_mask(T, mask_rate, 3)
    print("gpu ...", flush=True)
    dW = {k: to_dev(v, "bf16") for k, v in W.items()}
    drec = {k: to_dev(rec[k], "bf16") for k in REC}
    drec["LSE"] = torch.from_numpy(rec["LSE"]).cuda()
    out = A.alch_layer_backward(alch_shape(shp, "bf16"), A.Batch(cu), drec, dW, to_dev(dY, "bf16"),
                                loss_mask=None if mask is None else torch.from_numpy(mask).cuda())
    torch.cuda.synchronize()
    out = {k: v.float().cpu() for k, v in out.items()}      # free the device before the oracle takes the host
    del dW, drec
    torch.cuda.empty_cache()
    print("oracle ...", flush=True)
    ref = layer_backward_reuse(osh, cu, None, f64(rec), f64(W), dY.astype(np.float64), mask)
    return out, ref


def test_config2_full_size_every_output_elementwise():
    # config 2 as bench.py times it: Llama-3-8B-shaped layer, 4 x 2048 tokens; dX, the seven weight gradients
    # and both gain gradients, every element
    out, ref = _full_size_layer("llama8b", 4, 2048)
    assert set(out) == {"dX"} | {"d" + k for k in WEIGHT_KEYS}
    check_all(out, ref, 2e-2, "config2")


@pytest.mark.parametrize("mask_rate", [0.25, None])
def test_config5_full_size_every_output_elementwise(mask_rate):
    # config 5 as bench.py times it: Llama-3-70B-shaped layer, 2 x 4096 tokens, with the Bernoulli(0.25) loss mask
    # the configuration names (row-compacted path) and dense
    out, ref = _full_size_layer("llama70b", 2, 4096, mask_rate)
    check_all(out, ref, 2e-2, "config5 mask=%s" % mask_rate)


def test_config3_sized_capture_pack_one_layer():
    # 32 prompts with lengths U[256,4096], Bernoulli(0.25) keep mask, 6 streams out of fused buffers
    import paper_2503_01066_amd as A
    lens = synth.random_lengths(32, 256, 4096, 0)
    cu = synth.ragged_cu(lens)
    T = int(cu[-1])
    mask = synth.keep_mask(T, 0.25, 1)
    g = torch.Generator(device="cuda").manual_seed(0)
    hid = torch.randint(-2 ** 15, 2 ** 15, (T, 4096), generator=g, device="cuda", dtype=torch.int16)
    qkv = torch.randint(-2 ** 15, 2 ** 15, (T, 6144), generator=g, device="cuda", dtype=torch.int16)
    gu = torch.randint(-2 ** 15, 2 ** 15, (T, 28672), generator=g, device="cuda", dtype=torch.int16)
    streams = [hid, qkv[:, :4096], qkv[:, 4096:5120], qkv[:, 5120:], gu[:, :14336], gu[:, 14336:]]
    kept, cu_kept, status, dsts = A.alch_capture_pack(A.Batch(cu), torch.from_numpy(mask).cuda(), streams)
    torch.cuda.synchronize()
    ok, ocu, _ = gather_pack(mask, cu, [])
    n = len(ok)
    assert status.cpu().tolist() == [n, 0]
    assert np.array_equal(kept.cpu().numpy()[:n], ok) and np.array_equal(cu_kept.cpu().numpy(), ocu)
    # rows: sampled kept rows, each stream compared bit for bit with the source row the oracle index names
    rows = np.random.default_rng(2).choice(n, 64, replace=False)
    for s, d in zip(streams, dsts):
        src_rows = s[torch.from_numpy(ok[rows].astype(np.int64)).cuda()].cpu().numpy()
        assert np.array_equal(d[torch.from_numpy(rows).cuda()].cpu().numpy(), src_rows)
    # and every packed row equals its source row (checksum over all rows, on the device)
    idx = torch.from_numpy(ok.astype(np.int64)).cuda()
    for s, d in zip(streams, dsts):
        assert torch.equal(d[:n], s[idx])


def test_llama70b_width_short_batch_elementwise_with_loss_mask():
    # config-5 widths (hidden 8192, 64/8 heads x 128, ffn 28672), Bernoulli(0.25) loss mask, short ragged batch
    shp = synth.shape_dict("llama70b")
    osh = oracle_shape(shp)
    cu = synth.ragged_cu([70, 131])
    T = int(cu[-1])
    W = synth.layer_weights(shp, 0, "bf16")
    rec = synth.drawn_record(shp, T, 1, "bf16")
    rec["LSE"] = attention_lse(osh, cu, rec["Q"].astype(np.float64), rec["K"].astype(np.float64)).astype(np.float32)
    dY = synth.activations(T, shp["hidden"], 2, "bf16", std=0.01)
    mask = synth.keep_mask(T, 0.25, 3)
    print("oracle ...", flush=True)
    ref = layer_backward_reuse(osh, cu, None, f64(rec), f64(W), dY.astype(np.float64), mask)
    print("gpu ...", flush=True)
    import paper_2503_01066_amd as A
    dW = {k: to_dev(v, "bf16") for k, v in W.items()}
    drec = {k: to_dev(rec[k], "bf16") for k in REC}
    drec["LSE"] = torch.from_numpy(rec["LSE"]).cuda()
    out = A.alch_layer_backward(alch_shape(shp, "bf16"), A.Batch(cu), drec, dW, to_dev(dY, "bf16"),
                                loss_mask=torch.from_numpy(mask).cuda())
    torch.cuda.synchronize()
    for k, v in out.items():
        e = rel_err(to_np(v), ref[k])
        assert e <= 2e-2, (k, e)


def test_config2_full_size_adapter_mode_every_output_elementwise():
    # the paper's training setting at the size bench.py times (frozen 8B-shaped base, rank-8 adapters on all seven
    # projections, 4 x 2048 tokens): dX and all fourteen adapter gradients, every element
    import paper_2503_01066_amd as A
    from oracle.lora import layer_backward_reuse_lora
    shp = synth.shape_dict("llama8b")
    osh = oracle_shape(shp)
    S, B, r, scale = 2048, 4, 8, 2.0
    cu = synth.uniform_cu(B, S)
    T = B * S
    W = synth.layer_weights(shp, 0, "bf16")
    lora = synth.lora_adapters(shp, r, 5, "bf16", std=0.05)
    rec = synth.drawn_record(shp, T, 1, "bf16")
    print("lse ...", flush=True)
    rec["LSE"] = attention_lse(osh, cu, rec["Q"].astype(np.float64), rec["K"].astype(np.float64)).astype(np.float32)
    dY = synth.activations(T, shp["hidden"], 2, "bf16", std=0.01)
    print("gpu ...", flush=True)
    drec = {k: to_dev(rec[k], "bf16") for k in REC}
    drec["LSE"] = torch.from_numpy(rec["LSE"]).cuda()
    out = A.alch_layer_backward_lora(alch_shape(shp, "bf16"), A.Batch(cu), drec, {k: to_dev(v, "bf16") for k, v in W.items()},
                                     {p: (to_dev(a, "bf16"), to_dev(b, "bf16")) for p, (a, b) in lora.items()}, r, scale,
                                     to_dev(dY, "bf16"))
    torch.cuda.synchronize()
    out = {k: v.float().cpu() for k, v in out.items()}
    del drec
    torch.cuda.empty_cache()
    print("oracle ...", flush=True)
    lora64 = {p: (a.astype(np.float64), b.astype(np.float64)) for p, (a, b) in lora.items()}
    ref = layer_backward_reuse_lora(osh, cu, None, f64(rec), f64(W), lora64, scale, dY.astype(np.float64))
    assert {"dX"} | {"d" + m + p for p in lora for m in "AB"} <= set(out)
    check_all(out, ref, 2e-2, "config2 adapters")


def test_split_products_with_several_outputs_and_operand_pairs():
    # 2 x 512 tokens on a layer whose [dWq; dWk; dWv] product has 384 output tiles in three row ranges (its last round
    # of 128 tiles is split in two along the tokens) and whose data-gradient products have 32 tiles and up to three
    # operand pairs (every tile split): element-by-element against the oracle
    shp = synth.shape_dict("wideqkv")
    osh = oracle_shape(shp)
    cu = synth.ragged_cu([512, 512])
    T = 1024
    W = synth.layer_weights(shp, 7, "bf16", std=0.02, gain_std=0.1)
    rec = synth.drawn_record(shp, T, 8, "bf16")
    rec["LSE"] = attention_lse(osh, cu, rec["Q"].astype(np.float64), rec["K"].astype(np.float64)).astype(np.float32)
    dY = synth.activations(T, shp["hidden"], 9, "bf16", std=0.01)
    ref = layer_backward_reuse(osh, cu, None, f64(rec), f64(W), dY)
    out = gpu_layer(shp, cu, W, rec, dY)
    for k in ["dX"] + ["d" + w for w in WEIGHT_KEYS]:
        assert rel_err(to_np(out[k]), ref[k]) <= 2e-2, (k, rel_err(to_np(out[k]), ref[k]))
    # accumulate into gradients that already hold something: the finish kernel of a split product adds the old value
    import paper_2503_01066_amd as A
    rng = np.random.default_rng(3)
    scale = {k: float(np.abs(ref["d" + k]).max()) for k in WEIGHT_KEYS}
    old = {"d" + k: synth.quantize((rng.standard_normal(W[k].shape) * scale[k]).astype(np.float32), "bf16") for k in WEIGHT_KEYS}
    grads = {k: to_dev(v, "bf16") for k, v in old.items()}
    drec = {k: to_dev(rec[k], "bf16") for k in REC}
    drec["LSE"] = torch.from_numpy(rec["LSE"]).cuda()
    A.alch_layer_backward(alch_shape(shp, "bf16"), A.Batch(cu), drec, {k: to_dev(v, "bf16") for k, v in W.items()},
                          to_dev(dY, "bf16"), grads=grads, accumulate=True)
    torch.cuda.synchronize()
    for k in WEIGHT_KEYS:
        want = ref["d" + k] + old["d" + k].astype(np.float64)
        assert rel_err(to_np(grads["d" + k]), want) <= 2e-2, k


def test_shared_prompt_equals_duplicated_prefill_at_real_width():
    # Property that holds at any size (Section 4.1: chosen and rejected share the prompt's prefill): the DPO step on
    # [prompts | responses with a prefix] gives the loss and gradients of the step that prefills prompt + response
    # once per response.  Llama-3-8B-shaped layers, two prompts of 2048 and 700 tokens, responses of 128 tokens.
    import paper_2503_01066_amd as A
    dev, bf = "cuda", torch.bfloat16
    shp = synth.shape_dict("llama8b")
    shape = alch_shape(shp, "bf16")
    H, V, L, R = shp["hidden"], 4096, 2, 128
    prompts = [2048, 700]
    b = synth.preference_batch(prompts, [[R, R], [R, R]], V, 3)
    T, Tp = int(b["cu"][-1]), sum(prompts)
    g = torch.Generator(device=dev).manual_seed(1)
    rnd = lambda s_, std: (torch.randn(s_, generator=g, device=dev, dtype=torch.float32) * std).to(bf)
    QD, KD, F = shp["n_q_heads"] * shp["head_dim"], shp["n_kv_heads"] * shp["head_dim"], shp["ffn"]
    Ws = [{"Wq": rnd((QD, H), 0.02), "Wk": rnd((KD, H), 0.02), "Wv": rnd((KD, H), 0.02), "Wo": rnd((H, QD), 0.02),
           "Wg": rnd((F, H), 0.02), "Wu": rnd((F, H), 0.02), "Wd": rnd((H, F), 0.02),
           "g1": torch.ones(H, device=dev, dtype=bf), "g2": torch.ones(H, device=dev, dtype=bf)} for _ in range(L)]
    W_lm, g_final = rnd((V, H), 0.02), torch.ones(H, device=dev, dtype=bf)
    X0 = rnd((T, H), 1.0)
    ref = np.full(4, -R * np.log(V), np.float32)

    # shared: prompts first (as serving would), then the responses alone on their K/V
    batch = A.Batch(b["cu"], positions=b["positions"], prefix=b["prefix"])
    X, recs = X0, []
    for l in range(L):
        rec = {k: torch.empty((T, w), dtype=bf, device=dev) for k, w in dict(X=H, X2=H, Q=QD, K=KD, V=KD, O=QD, G=F, U=F).items()}
        rec["LSE"] = torch.empty((T, shp["n_q_heads"]), dtype=torch.float32, device=dev)
        Y, rec = A.alch_layer_forward(shape, A.Batch(b["cu"][:3]), X, Ws[l], rec=rec, Y=torch.empty((T, H), dtype=bf, device=dev))
        A.alch_layer_forward(shape, batch, X, Ws[l], seq_begin=2, rec=rec, Y=Y)
        recs.append(rec)
        X = Y
    out = A.alch_stack_backward_dpo(shape, batch, recs, Ws, X, g_final, W_lm, b["item_row"], b["item_label"], b["item_slot"], ref, 0.1)

    # duplicated: [prompt; response] per response
    lens = [prompts[0] + R, prompts[0] + R, prompts[1] + R, prompts[1] + R]
    cu_d = synth.ragged_cu(lens)
    src, rows, labels, slots = [], [], [], []
    tok = b["tokens"]
    for k in range(4):
        gq = k // 2
        p0 = int(b["cu"][gq])
        src += list(range(p0, p0 + prompts[gq])) + list(range(Tp + k * R, Tp + (k + 1) * R))
        a = int(cu_d[k])
        rows += list(range(a + prompts[gq] - 1, a + prompts[gq] + R - 1))
        labels += list(tok[Tp + k * R: Tp + (k + 1) * R])
        slots += [k] * R
    src_t = torch.tensor(src, device=dev)
    batch_d = A.Batch(cu_d)
    Xd, recs_d = X0[src_t], []
    for l in range(L):
        Xd, rec = A.alch_layer_forward(shape, batch_d, Xd, Ws[l])
        recs_d.append(rec)
    out_d = A.alch_stack_backward_dpo(shape, batch_d, recs_d, Ws, Xd, g_final, W_lm, np.asarray(rows, np.int32),
                                      np.asarray(labels, np.int32), np.asarray(slots, np.int32), ref, 0.1)
    torch.cuda.synchronize()

    # (700 is no multiple of the 64-key tile: the two paths split the softmax sums differently, so they agree to
    # bf16 rounding of the logits, not bit for bit)
    assert abs(out["loss"].item() - out_d["loss"].item()) <= 2e-2 * max(1.0, abs(out_d["loss"].item()))
    assert rel_err(to_np(out["z"]), to_np(out_d["z"])) <= 2e-2
    # gradient w.r.t. the embeddings: duplicated rows of a prompt add up
    want = torch.zeros((T, H), dtype=torch.float32, device=dev)
    want.index_add_(0, src_t, out_d["dX_embed"].float())
    assert rel_err(to_np(out["dX_embed"]), to_np(want)) <= 2e-2
    assert float(out["dX_embed"][:Tp].abs().max()) > 0
    for k in ("dW_lm", "dg_final"):
        assert rel_err(to_np(out[k]), to_np(out_d[k])) <= 2e-2, k
    for l in range(L):
        for k in out["layers"][l]:
            e = rel_err(to_np(out["layers"][l][k]), to_np(out_d["layers"][l][k]))
            assert e <= 2e-2, (l, k, e)
