"""The hot path is allocation-free and stream-ordered, so it can be captured in a HIP graph; its
kernels use no atomics, so results are bit-reproducible.  Replays are checked against the eager
result, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import synth_inputs as synth
from helpers import to_dev, alch_shape

pytestmark = pytest.mark.gpu
REC = ("X", "X2", "Q", "K", "V", "O", "G", "U")


def setup_case():
    import paper_2503_01066_amd as A
    shp = synth.shape_dict("medium")
    lens, keep = [200, 96, 130], [1, 0, 1]
    cu = synth.ragged_cu(lens)
    T = int(cu[-1])
    W = {k: to_dev(v, "bf16") for k, v in synth.layer_weights(shp, 0, "bf16").items()}
    src = {k: to_dev(v, "bf16") for k, v in synth.drawn_record(shp, T, 1, "bf16").items()}
    src["LSE"] = torch.from_numpy(np.random.default_rng(2).normal(6.0, 0.3, (T, shp["n_q_heads"])).astype(np.float32)).cuda()
    mask = torch.from_numpy(np.concatenate([np.full(n, k, np.uint8) for n, k in zip(lens, keep)])).cuda()
    kept_lens = [n for n, k in zip(lens, keep) if k]
    Tk = sum(kept_lens)
    dY = to_dev(synth.activations(Tk, shp["hidden"], 3, "bf16", std=0.01), "bf16")
    shape = alch_shape(shp, "bf16")
    keys = list(REC) + ["LSE"]
    dst = {k: torch.empty((Tk, src[k].shape[1]), dtype=src[k].dtype, device="cuda") for k in keys}
    grads = {"d" + k: torch.empty_like(v) for k, v in W.items()}
    dX = torch.empty_like(dY)
    src_batch, kept_batch = A.Batch(cu), A.Batch(synth.ragged_cu(kept_lens))
    ws_pack = torch.empty(A.lib().alch_capture_pack_workspace_bytes(T), dtype=torch.uint8, device="cuda")
    ws = torch.empty(A.layer_backward_workspace_bytes(shape, Tk, max(kept_lens)), dtype=torch.uint8, device="cuda")

    def step():
        A.alch_capture_pack(src_batch, mask, [src[k] for k in keys], capacity=Tk, dsts=[dst[k] for k in keys],
                            workspace=ws_pack)
        A.alch_layer_backward(shape, kept_batch, dst, W, dY, grads=grads, dX=dX, workspace=ws)

    outs = dict(grads, dX=dX)
    return step, outs, src


def snapshot(outs):
    torch.cuda.synchronize()
    return {k: v.clone() for k, v in outs.items()}


def test_bit_reproducible():
    step, outs, _ = setup_case()
    step()
    a = snapshot(outs)
    for v in outs.values():
        v.zero_()
    step()
    b = snapshot(outs)
    for k in a:
        assert torch.equal(a[k], b[k]), k


def test_graph_replays_match_eager():
    step, outs, src = setup_case()
    step()
    eager = snapshot(outs)
    # kept_index / status tensors are allocated by the binding: warm the allocator on a side stream, then capture
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(3):
        for v in outs.values():
            v.fill_(float(rep))           # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        got = snapshot(outs)
        for k in eager:
            assert torch.equal(got[k], eager[k]), (rep, k)
    # a replay sees new input values (same addresses): scale dO-side input and compare with eager again
    src["G"].mul_(0.5)
    torch.cuda.synchronize()
    g.replay()
    got = snapshot(outs)
    step()
    again = snapshot(outs)
    for k in again:
        assert torch.equal(got[k], again[k]), k


def test_graph_with_loss_mask_compaction_and_adapters():
    # the row count of the loss-mask mode lives on the device: a captured graph must follow a mask whose
    # contents change between replays (same address); the adapter mode is captured in the same graph
    import paper_2503_01066_amd as A
    shp = synth.shape_dict("medium")
    cu = synth.ragged_cu([200, 96, 130])
    T = int(cu[-1])
    shape = alch_shape(shp, "bf16")
    batch = A.Batch(cu)
    W = {k: to_dev(v, "bf16") for k, v in synth.layer_weights(shp, 0, "bf16").items()}
    rec = {k: to_dev(v, "bf16") for k, v in synth.drawn_record(shp, T, 1, "bf16").items()}
    rec["LSE"] = torch.from_numpy(np.random.default_rng(2).normal(6.0, 0.3, (T, shp["n_q_heads"])).astype(np.float32)).cuda()
    dY = to_dev(synth.activations(T, shp["hidden"], 3, "bf16", std=0.01), "bf16")
    mask = torch.from_numpy(synth.keep_mask(T, 0.3, 1)).cuda()
    lora = {p: (to_dev(a, "bf16"), to_dev(b, "bf16")) for p, (a, b) in synth.lora_adapters(shp, 8, 4, "bf16").items()}
    grads = {"d" + k: torch.empty_like(v) for k, v in W.items()}
    lgrads = {}
    for p, (a, b) in lora.items():
        lgrads["dA" + p], lgrads["dB" + p] = torch.empty_like(a), torch.empty_like(b)
    dX1, dX2 = torch.empty_like(dY), torch.empty_like(dY)
    import ctypes
    ws1 = torch.empty(A.layer_backward_workspace_bytes(shape, T, 200), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(A.lib().alch_layer_backward_lora_workspace_bytes(ctypes.byref(shape), T, 200, 8), dtype=torch.uint8,
                      device="cuda")

    def step():
        A.alch_layer_backward(shape, batch, rec, W, dY, loss_mask=mask, grads=grads, dX=dX1, workspace=ws1)
        A.alch_layer_backward_lora(shape, batch, rec, W, lora, 8, 2.0, dY, lora_grads=lgrads, dX=dX2, workspace=ws2)

    outs = dict(grads, dX1=dX1, dX2=dX2, **lgrads)
    step()
    eager = snapshot(outs)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(2):
        for v in outs.values():
            v.fill_(float(rep))
        torch.cuda.synchronize()
        g.replay()
        got = snapshot(outs)
        for k in eager:
            assert torch.equal(got[k], eager[k]), (rep, k)
    mask.copy_(torch.from_numpy(synth.keep_mask(T, 0.7, 9)).cuda())   # other rows, another count
    torch.cuda.synchronize()
    g.replay()
    got = snapshot(outs)
    step()
    again = snapshot(outs)
    assert not torch.equal(again["dWd"], eager["dWd"])
    for k in again:
        assert torch.equal(got[k], again[k]), k


def test_graph_of_the_preference_alignment_step():
    # forward of the responses alone on the prompts' saved K/V + DPO head + backward through the shared prompt,
    # captured once; replays follow new response embeddings written to the same addresses
    import paper_2503_01066_amd as A
    shp = synth.shape_dict("medium")
    shape = alch_shape(shp, "bf16")
    H, V, L = shp["hidden"], 512, 2
    b = synth.preference_batch([150, 70], [[60, 33], [129, 20]], V, 2)
    T, n_p = int(b["cu"][-1]), int(b["cu"][2])
    batch = A.Batch(b["cu"], positions=b["positions"], prefix=b["prefix"])
    Ws = [{k: to_dev(v, "bf16") for k, v in synth.layer_weights(shp, 10 * l, "bf16", std=0.05).items()} for l in range(L)]
    rng = np.random.default_rng(3)
    Wlm, gf = to_dev(synth.normal(rng, (V, H), 0.05, "bf16"), "bf16"), torch.ones(H, dtype=torch.bfloat16, device="cuda")
    acts = [to_dev(synth.normal(rng, (T, H), 1.0, "bf16"), "bf16")] + [torch.empty((T, H), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
    QD, KD, F = shp["n_q_heads"] * shp["head_dim"], shp["n_kv_heads"] * shp["head_dim"], shp["ffn"]
    recs = []
    for l in range(L):   # the prompts' rows: the serving prefill
        rec = {k: torch.empty((T, w), dtype=torch.bfloat16, device="cuda") for k, w in dict(X2=H, Q=QD, K=KD, V=KD, O=QD, G=F, U=F).items()}
        rec["X"] = acts[l]
        rec["LSE"] = torch.empty((T, shp["n_q_heads"]), dtype=torch.float32, device="cuda")
        A.alch_layer_forward(shape, A.Batch(b["cu"][:3]), acts[l], Ws[l], rec=rec, Y=acts[l + 1])
        recs.append(rec)
    items = A.DpoItems(b["item_row"], b["item_label"], b["item_slot"], rng.normal(-3, 1, 4).astype(np.float32))
    grads = [{"d" + k: torch.empty_like(v) for k, v in W.items()} for W in Ws]
    ws = torch.empty(A.stack_backward_workspace_bytes(shape, L, V, T, 150), dtype=torch.uint8, device="cuda")
    import ctypes
    ws_f = torch.empty(A.lib().alch_layer_forward_workspace_bytes(ctypes.byref(shape), T, 150), dtype=torch.uint8, device="cuda")
    holder = {}

    def step():
        for l in range(L):
            A.alch_layer_forward(shape, batch, acts[l], Ws[l], workspace=ws_f, seq_begin=2, rec=recs[l], Y=acts[l + 1])
        holder["out"] = A.alch_stack_backward_dpo(shape, batch, recs, Ws, acts[L], gf, Wlm, items, None, None, None, 0.5,
                                                  grads_layers=grads, workspace=ws)

    def outputs():
        o = holder["out"]
        d = {"loss": o["loss"], "z": o["z"], "dX_embed": o["dX_embed"], "dW_lm": o["dW_lm"]}
        for l in range(L):
            d.update({"%d.%s" % (l, k): v for k, v in grads[l].items()})
        return d

    step()
    eager = snapshot(outputs())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(2):
        for v in outputs().values():
            v.fill_(float(rep))
        torch.cuda.synchronize()
        g.replay()
        got = snapshot(outputs())
        for k in eager:
            assert torch.equal(got[k], eager[k]), (rep, k)
    acts[0][n_p:].mul_(0.5)      # other responses at the same addresses
    torch.cuda.synchronize()
    g.replay()
    got = snapshot(outputs())
    step()
    again = snapshot(outputs())
    assert not torch.equal(again["loss"], eager["loss"])
    for k in again:
        assert torch.equal(got[k], again[k]), k
