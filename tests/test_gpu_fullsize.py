"""Full-size parity in the launch configuration bench.py times (config 2: one Llama-3-8B-shaped
layer, bf16, 4 x 2048 tokens), on sampled outputs the oracle can compute one by one, plus a
full-width / short-batch case checked element by element, plus config-3-sized capture/pack."""
import numpy as np
import pytest
import torch

import synth_inputs as synth
from helpers import to_dev, to_np, f64, rel_err, oracle_shape, alch_shape
from oracle import layer_backward_reuse, attention_lse, gather_pack, WEIGHT_KEYS
from oracle.layer import layer_backward_reuse_tail_rows, _rms_norm, _sigmoid

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


def test_config2_full_size_sampled_outputs():
    shp = synth.shape_dict("llama8b")
    osh = oracle_shape(shp)
    S, B = 2048, 4
    cu = synth.uniform_cu(B, S)
    T = B * S
    H, F = shp["hidden"], shp["ffn"]
    W = synth.layer_weights(shp, 0, "bf16")
    rec = synth.drawn_record(shp, T, 1, "bf16")
    print("lse ...", flush=True)
    rec["LSE"] = attention_lse(osh, cu, rec["Q"].astype(np.float64), rec["K"].astype(np.float64)).astype(np.float32)
    dY = synth.activations(T, H, 2, "bf16", std=0.01)
    print("gpu ...", flush=True)
    out = gpu_layer(shp, cu, W, rec, dY)
    W64 = f64(W)
    rng = np.random.default_rng(3)

    # (a) dX rows of the last tokens of two sequences (exact by causality)
    m = 24
    dX = to_np(out["dX"])
    for s in (0, 3):
        a, b = s * S, (s + 1) * S
        seq = {k: rec[k][a:b].astype(np.float64) for k in REC + ("LSE",)}
        tail = layer_backward_reuse_tail_rows(osh, None, seq, W64, dY[b - m:b].astype(np.float64))
        e = np.abs(dX[b - m:b] - tail).max() / np.abs(tail).max()
        assert e <= 2e-2, ("dX tail", s, e)

    # (b) sampled entries of dWd = dY^T (silu(G) * U)
    dWd = to_np(out["dWd"])
    G64, U64, dY64 = rec["G"].astype(np.float64), rec["U"].astype(np.float64), dY.astype(np.float64)
    oo, ii = rng.integers(0, H, 48), rng.integers(0, F, 48)
    want = np.array([np.sum(dY64[:, o] * (G64[:, i] * _sigmoid(G64[:, i]) * U64[:, i])) for o, i in zip(oo, ii)])
    scale = np.abs(want).max()
    assert np.abs(dWd[oo, ii] - want).max() <= 2e-2 * scale

    # (c) sampled entries of dWg, dWu = dG^T H2, dU^T H2 with dAct[:, f] = dY Wd[:, f]
    X2 = rec["X2"].astype(np.float64)
    H2, _ = _rms_norm(X2, W64["g2"], osh.rms_eps)
    dWg, dWu = to_np(out["dWg"]), to_np(out["dWu"])
    ff, hh = rng.integers(0, F, 12), rng.integers(0, H, 12)
    wg, wu = [], []
    for f, h in zip(ff, hh):
        dAct = dY64 @ W64["Wd"][:, f]
        sg = _sigmoid(G64[:, f])
        wg.append(np.sum(dAct * U64[:, f] * sg * (1 + G64[:, f] * (1 - sg)) * H2[:, h]))
        wu.append(np.sum(dAct * G64[:, f] * sg * H2[:, h]))
    wg, wu = np.array(wg), np.array(wu)
    # the bar is relative to the largest entry of the tensor; the samples give a lower bound of it
    assert np.abs(dWg[ff, hh] - wg).max() <= 2e-2 * max(np.abs(wg).max(), np.abs(dWg).max())
    assert np.abs(dWu[ff, hh] - wu).max() <= 2e-2 * max(np.abs(wu).max(), np.abs(dWu).max())
    for k, v in out.items():
        assert torch.isfinite(v.float()).all(), k


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


def test_config2_full_size_adapter_mode_sampled_outputs():
    # the paper's training setting at the size bench.py times (frozen 8B-shaped base, rank-8 adapters on all seven
    # projections, 4 x 2048 tokens): dX rows by causality at the merged weights, sampled adapter-gradient entries
    # from their definitions
    import paper_2503_01066_amd as A
    from oracle.lora import merged_weights
    shp = synth.shape_dict("llama8b")
    osh = oracle_shape(shp)
    S, B, r, scale = 2048, 4, 8, 2.0
    cu = synth.uniform_cu(B, S)
    T = B * S
    H, F = shp["hidden"], shp["ffn"]
    W = synth.layer_weights(shp, 0, "bf16")
    lora = synth.lora_adapters(shp, r, 5, "bf16", std=0.05)
    rec = synth.drawn_record(shp, T, 1, "bf16")
    print("lse ...", flush=True)
    rec["LSE"] = attention_lse(osh, cu, rec["Q"].astype(np.float64), rec["K"].astype(np.float64)).astype(np.float32)
    dY = synth.activations(T, H, 2, "bf16", std=0.01)
    print("gpu ...", flush=True)
    drec = {k: to_dev(rec[k], "bf16") for k in REC}
    drec["LSE"] = torch.from_numpy(rec["LSE"]).cuda()
    out = A.alch_layer_backward_lora(alch_shape(shp, "bf16"), A.Batch(cu), drec, {k: to_dev(v, "bf16") for k, v in W.items()},
                                     {p: (to_dev(a, "bf16"), to_dev(b, "bf16")) for p, (a, b) in lora.items()}, r, scale,
                                     to_dev(dY, "bf16"))
    torch.cuda.synchronize()
    lora64 = {p: (a.astype(np.float64), b.astype(np.float64)) for p, (a, b) in lora.items()}
    Wm = merged_weights(f64(W), lora64, scale)
    rng = np.random.default_rng(4)

    # (a) dX rows of the last tokens of a sequence (exact by causality), merged weights
    m = 16
    dX = to_np(out["dX"])
    a, b = 2 * S, 3 * S
    seq = {k: rec[k][a:b].astype(np.float64) for k in REC + ("LSE",)}
    tail = layer_backward_reuse_tail_rows(osh, None, seq, Wm, dY[b - m:b].astype(np.float64))
    e = np.abs(dX[b - m:b] - tail).max() / np.abs(tail).max()
    assert e <= 2e-2, ("dX tail", e)

    # (b) down-projection adapter: dB_d = s dY^T (Act A_d^T), dA_d = s (dY B_d)^T Act, all entries of the small matrices
    G64, U64, dY64 = rec["G"].astype(np.float64), rec["U"].astype(np.float64), dY.astype(np.float64)
    Act = G64 * _sigmoid(G64) * U64
    Ad, Bd = lora64["d"]
    want_dB = scale * dY64.T @ (Act @ Ad.T)
    want_dA = scale * (dY64 @ Bd).T @ Act
    assert rel_err(to_np(out["dBd"]), want_dB) <= 2e-2
    assert rel_err(to_np(out["dAd"]), want_dA) <= 2e-2

    # (c) gate adapter, sampled columns f: dG[:, f] from dAct[:, f] = dY Wd'[:, f]; dB_g[f, :] = s dG[:, f]^T (H2 A_g^T)
    H2, _ = _rms_norm(rec["X2"].astype(np.float64), Wm["g2"], osh.rms_eps)
    Ag, Bg = lora64["g"]
    t1 = scale * (H2 @ Ag.T)
    dBg = to_np(out["dBg"])
    ff = rng.integers(0, F, 10)
    want = []
    for f in ff:
        dAct = dY64 @ Wm["Wd"][:, f]
        sg = _sigmoid(G64[:, f])
        want.append((dAct * U64[:, f] * sg * (1 + G64[:, f] * (1 - sg))) @ t1)
    want = np.array(want)
    assert np.abs(dBg[ff] - want).max() <= 2e-2 * max(np.abs(want).max(), np.abs(dBg).max())
    for k, v in out.items():
        assert torch.isfinite(v.float()).all(), k


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
