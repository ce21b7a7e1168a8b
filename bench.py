#!/usr/bin/env python3
"""Benchmark of the activation-reuse hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic batch:
  capture/pack of a layer's saved activations (mask scan + row gather of the 9 record
  streams, keeping 4 of 16 prefilled prompts) followed by the decoder-layer backward pass
  driven by the packed record (all data and weight gradients).
Workload "config2" (default): one Llama-3-8B-shaped layer, bf16, hidden 4096, 32 Q / 8 KV heads
x 128, FFN 14336; the trained batch is 4 sequences x 2048 tokens.
Workload "config3": capture/pack only, 32 layers x 32 prompts with lengths in [256, 4096],
per-token keep mask ~ Bernoulli(0.25), 6 streams per layer out of fused qkv / gate-up buffers.

Prints ONE JSON line (see the keys below).  Inputs are resident in HBM before timing starts.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "backward training tokens/sec from reused activations; capture GB/s; % roofline"
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="config2", choices=["config2", "config3", "config4", "config5", "dpo", "short", "copy", "gemm"])
    ap.add_argument("--layers", type=int, default=32, help="config4: number of layers")
    ap.add_argument("--loss-mask", action="store_true", help="config5: zero dY rows with a Bernoulli(0.25) loss mask")
    ap.add_argument("--lora-rank", type=int, default=0,
                    help="config2/config5: rank-r adapters on all seven projections (alch_layer_backward_lora)")
    ap.add_argument("--frozen-base", action="store_true",
                    help="config2/config5: no base weight gradients (the frozen base of parameter-efficient fine-tuning)")
    ap.add_argument("--offload", action="store_true",
                    help="config4: records live in pinned host memory and are prefetched layer by layer during the walk")
    ap.add_argument("--six-stream", action="store_true",
                    help="pack / keep only X, Q, K, V, G, U; the backward recomputes O, LSE and X2")
    ap.add_argument("--four-stream", action="store_true",
                    help="pack / keep only X, Q, K, V; the backward recomputes O, LSE, X2, G and U")
    ap.add_argument("--scan-once", action="store_true",
                    help="config3: scan the mask for the first layer only, alch_capture_gather for the other 31")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-full", action="store_true",
                    help="time the oracle on the whole workload (config 3: all 32 layers; config 5: 2 x 4096 tokens) "
                         "instead of the bounded sample; takes several minutes of host time")
    ap.add_argument("--headline-only", action="store_true",
                    help="config2: leave out the `also` object (configs 3, 4 and 5 measured in the same run)")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "traffic.json"),
                    help="measured HBM bytes per launch (from the rocprofv3 --pmc summaries)")
    return ap.parse_args()


def cpu_baseline_layer(workload, seed=0, full=False):
    """The fp64 oracle, as it stands, on a bounded sample of the layer workload (full: on all of it)."""
    import synth_inputs as synth
    from oracle import LayerShape, layer_backward_reuse, attention_lse
    shape_name = LAYER_WORKLOADS[workload][0]
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    shp = synth.shape_dict(shape_name)
    osh = LayerShape(*[shp[k] for k in synth.SHAPE_FIELDS])
    # a bounded sample (10-30 s of host time): config 2 in full (4 x 2048); of config 5, one sequence of 2048 tokens
    # (the whole 2 x 4096 with full=True, about two minutes)
    n_seq, S = (4, 2048) if workload == "config2" else ((1, 512) if workload == "short" else ((2, 4096) if full else (1, 2048)))
    cu = np.arange(n_seq + 1) * S
    Ttot = n_seq * S
    W = {k: v.astype(np.float64) for k, v in synth.layer_weights(shp, seed, "bf16").items()}
    rec = {k: v.astype(np.float64) for k, v in synth.drawn_record(shp, Ttot, seed + 1, "bf16").items()}
    dY = synth.activations(Ttot, shp["hidden"], seed + 2, "bf16", std=0.01).astype(np.float64)
    t0 = time.perf_counter()
    rec["LSE"] = attention_lse(osh, cu, rec["Q"], rec["K"])
    layer_backward_reuse(osh, cu, None, rec, W, dY)
    dt = time.perf_counter() - t0
    return {"value": Ttot / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d sequences of %d tokens of the same %s-shaped layer (all nine gradients), fp64 numpy, %.1f s"
                      % (n_seq, S, shape_name, dt)}


def cpu_baseline_dpo(layers, seed=0):
    """The shared-prefix oracle, as it stands, on a bounded sample of the dpo workload: one layer of the same shape,
    one prompt of 1024 tokens with two responses of 128 tokens (response rows forward + layer backward); the
    figure is scaled to the stack by the layer count and labelled so."""
    import synth_inputs as synth
    from oracle import LayerShape
    from oracle.prefix import layer_forward_prefix, layer_backward_reuse_prefix
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    shp = synth.shape_dict("llama8b")
    osh = LayerShape(*[shp[k] for k in synth.SHAPE_FIELDS])
    b = synth.preference_batch([1024], [[128, 128]], 1000, seed)
    T = int(b["cu"][-1])
    W = {k: v.astype(np.float64) for k, v in synth.layer_weights(shp, seed, "bf16").items()}
    X = synth.activations(T, shp["hidden"], seed + 1, "bf16").astype(np.float64)
    dY = synth.activations(T, shp["hidden"], seed + 2, "bf16", std=0.01).astype(np.float64)
    _, rec = layer_forward_prefix(osh, b["cu"], b["prefix"], X, W)     # untimed: the serving prefill
    t0 = time.perf_counter()
    # the oracle has no response-only forward: the whole-batch forward is timed and charged by the response share
    layer_forward_prefix(osh, b["cu"], b["prefix"], X, W)
    t_fwd = (time.perf_counter() - t0) * 256.0 / T
    t1 = time.perf_counter()
    layer_backward_reuse_prefix(osh, b["cu"], b["prefix"], rec, W, dY)
    dt = t_fwd + time.perf_counter() - t1
    return {"value": T / dt / layers, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "EXTRAPOLATED to %d layers (LM head left out) from one llama8b-shaped layer on 1 prompt x 1024 + 2 "
                      "responses x 128 tokens: response share of the forward + full backward, fp64 numpy, %.1f s" % (layers, dt)}


def cpu_baseline_config3(seed=0, layers=4):
    """The gather oracle, as it stands, on the config-3 batch for a bounded number of layers."""
    import synth_inputs as synth
    from oracle import gather_pack
    lens = synth.random_lengths(32, 256, 4096, seed)
    cu = synth.ragged_cu(lens)
    T = int(cu[-1])
    mask = synth.keep_mask(T, 0.25, seed + 1)
    widths = (4096, 4096, 1024, 1024, 14336, 14336)
    # contents do not matter for the timing; one source set serves every layer of the sample
    srcs = [np.full((T, w), 0x3c00 + i, dtype=np.uint16) for i, w in enumerate(widths)]
    t0 = time.perf_counter()
    nbytes = 0
    for _ in range(layers):
        kept, _, packed = gather_pack(mask, cu, srcs)
        nbytes += 2 * sum(p.nbytes for p in packed)
    dt = time.perf_counter() - t0
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "%d of the 32 layers of the same batch (%d tokens, %d kept per layer), python/numpy row loop, "
                      "%.1f s" % (layers, T, len(kept), dt)}


def load_traffic(path, key):
    try:
        with open(path) as f:
            return json.load(f).get(key)
    except Exception:
        return None


LAYER_WORKLOADS = {
    # name: (shape, prefilled prompts, tokens per prompt, prompts kept for training, description)
    "config2": ("llama8b", 16, 2048, 4, "config2: one Llama-3-8B-shaped layer, bf16, 4 x 2048 trained tokens "
                "(packed out of 16 x 2048 prefilled), capture/pack + full layer backward"),
    "config5": ("llama70b", 8, 4096, 2, "config5: one Llama-3-70B-shaped layer, bf16, 2 x 4096 trained tokens "
                "(packed out of 8 x 4096 prefilled), capture/pack + full layer backward"),
    # per-query training right after serving (Section 4.4 of the paper caches one query of a batch): a short batch,
    # whose products have too few output tiles to fill the chip unless they are split along the contraction
    "short": ("llama8b", 4, 512, 1, "short: one Llama-3-8B-shaped layer, bf16, 1 x 512 trained tokens "
              "(packed out of 4 x 512 prefilled), capture/pack + full layer backward"),
}


def run_layer(args, torch, A):
    import synth_inputs as synth
    dev = "cuda"
    shape_name, n_src, S, n_keep, descr = LAYER_WORKLOADS[args.workload]
    shp = synth.shape_dict(shape_name)
    shape = A.make_shape(*[shp[k] for k in synth.SHAPE_FIELDS], "bf16")
    H, QD, KD, F = shp["hidden"], shp["n_q_heads"] * shp["head_dim"], shp["n_kv_heads"] * shp["head_dim"], shp["ffn"]
    T_src, T = n_src * S, n_keep * S
    g = torch.Generator(device=dev).manual_seed(0)
    bf = torch.bfloat16
    rnd = lambda shape_, std: (torch.randn(shape_, generator=g, device=dev, dtype=torch.float32) * std).to(bf)

    # prefill-side buffers of 16 prompts (the serving batch), record streams ~ N(0,1)
    widths = dict(X=H, X2=H, Q=QD, K=KD, V=KD, O=QD, G=F, U=F)
    src = {k: rnd((T_src, w), 1.0) for k, w in widths.items()}
    rs = np.random.default_rng(0)
    keep_seqs = np.sort(rs.choice(n_src, n_keep, replace=False))
    mask_np = np.zeros(T_src, np.uint8)
    for s in keep_seqs:
        mask_np[s * S:(s + 1) * S] = 1
    mask = torch.from_numpy(mask_np).to(dev)
    # LSE of the kept prompts from their own Q, K (attention forward of the library)
    src["LSE"] = torch.zeros((T_src, shp["n_q_heads"]), dtype=torch.float32, device=dev)
    one = A.Batch(synth.uniform_cu(1, S))
    for s in keep_seqs:
        sl = slice(int(s) * S, int(s + 1) * S)
        _, lse = A.alch_attention_forward(shape, one, src["Q"][sl], src["K"][sl], src["V"][sl])
        src["LSE"][sl] = lse
    W = {"Wq": rnd((QD, H), 0.02), "Wk": rnd((KD, H), 0.02), "Wv": rnd((KD, H), 0.02), "Wo": rnd((H, QD), 0.02),
         "Wg": rnd((F, H), 0.02), "Wu": rnd((F, H), 0.02), "Wd": rnd((H, F), 0.02),
         "g1": torch.ones(H, device=dev, dtype=bf), "g2": torch.ones(H, device=dev, dtype=bf)}
    dY = rnd((T, H), 0.01)
    loss_mask = None
    if args.loss_mask:
        lm_np = synth.keep_mask(T, 0.25, 7)
        n_loss = int(lm_np.sum())
        loss_mask = torch.from_numpy(lm_np).to(dev)
        descr += (", dY rows zeroed by a Bernoulli(0.25) loss mask (%d of %d rows kept): the row-local products run on "
                  "the kept rows, attention and the QKV products stay dense" % (n_loss, T))

    keys = list(widths) + ["LSE"]
    if args.six_stream:
        keys = ["X", "Q", "K", "V", "G", "U"]
        descr += ", six-stream record (O, LSE, X2 recomputed by the backward)"
    if args.four_stream:
        keys = ["X", "Q", "K", "V"]
        descr += ", four-stream record (O, LSE, X2, G, U recomputed by the backward)"
    dst = {k: torch.empty((T, src[k].shape[1]), dtype=src[k].dtype, device=dev) for k in keys}
    src_batch = A.Batch(synth.uniform_cu(n_src, S))
    kept_batch = A.Batch(synth.uniform_cu(n_keep, S))
    grads = {} if args.frozen_base else {"d" + k: torch.empty_like(v) for k, v in W.items()}
    dX = torch.empty_like(dY)
    ws_pack = torch.empty(A.lib().alch_capture_pack_workspace_bytes(T_src), dtype=torch.uint8, device=dev)
    streams = [src[k] for k in keys]
    dsts = [dst[k] for k in keys]
    r = args.lora_rank
    wflops = 2.0 if args.frozen_base else 4.0   # GEMM flops per parameter and token
    if args.frozen_base:
        descr += ", frozen base (data-gradient products only)"
    if r:
        import ctypes
        dims = dict(q=(QD, H), k=(KD, H), v=(KD, H), o=(H, QD), g=(F, H), u=(F, H), d=(H, F))
        lora = {p: (rnd((r, i), 0.05), rnd((o, r), 0.05)) for p, (o, i) in dims.items()}
        lgrads = {}
        for p, (a, b) in lora.items():
            lgrads["dA" + p], lgrads["dB" + p] = torch.empty_like(a), torch.empty_like(b)
        need = A.lib().alch_layer_backward_lora_workspace_bytes(ctypes.byref(shape), T, S, r)
        ws_bwd = torch.empty(need, dtype=torch.uint8, device=dev)
        descr += ", rank-%d adapters on all seven projections" % r

        def step():
            A.alch_capture_pack(src_batch, mask, streams, capacity=T, dsts=dsts, workspace=ws_pack)
            A.alch_layer_backward_lora(shape, kept_batch, dst, W, lora, r, 2.0, dY, loss_mask=loss_mask, grads=grads,
                                       lora_grads=lgrads, dX=dX, workspace=ws_bwd)
    else:
        ws_bwd = torch.empty(A.layer_backward_workspace_bytes(shape, T, S), dtype=torch.uint8, device=dev)

        def step():
            A.alch_capture_pack(src_batch, mask, streams, capacity=T, dsts=dsts, workspace=ws_pack)
            A.alch_layer_backward(shape, kept_batch, dst, W, dY, loss_mask=loss_mask, grads=grads, dX=dX, workspace=ws_bwd)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    A.alch_trace_enable(True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]  # step boundaries, current stream
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    A.alch_trace_enable(False)
    trace = A.alch_trace_collect()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    # the same K steps once more with the launch trace off (no event creation / recording in the loop)
    t1 = time.perf_counter()
    for i in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_untraced = (time.perf_counter() - t1) / args.steps * 1e3

    ms_step = dt / args.steps * 1e3
    by = {}
    for kind, flops, nbytes, ms in trace:
        e = by.setdefault(kind, [0.0, 0.0, 0.0, 0])
        e[0] += flops; e[1] += nbytes; e[2] += ms; e[3] += 1
    gm = by.get("gemm_mfma", [0, 0, 1e-9, 1])
    P = 2 * H * QD + 2 * H * KD + 3 * H * F
    gemm_flops_step = wflops * P * T
    if args.loss_mask and not r:
        # products whose row count lives on the device are traced without flops: count what the method must touch
        p_rows = 3 * H * F + H * QD                    # Wd, Wg, Wu, Wo: row-local, run on the kept rows
        gemm_flops_step = wflops * (p_rows * n_loss + (P - p_rows) * T)
        gm[0] = gemm_flops_step * args.steps
    achieved_tf = gm[0] / (gm[2] * 1e-3) / 1e12
    pk = by.get("pack_gather", [0, 0, 1e-9, 1])
    pack_gbps = pk[1] * T / (pk[2] * 1e-3) / 1e9       # traced bytes are per kept row
    attn_flops = 10.0 * shp["head_dim"] * shp["n_q_heads"] * n_keep * S * (S + 1) / 2
    kms = {k: v[2] / args.steps for k, v in by.items()}
    pack_ms = kms.get("pack_scan", 0.0) + kms.get("pack_gather", 0.0)
    bwd_ms = ms_step - pack_ms                         # the layer backward alone: the step minus the capture/pack call
    attn_ms = kms.get("attn_bwd", 0.0)
    row_bytes_rw = pk[1] / max(pk[3], 1)                # traced bytes of a gather launch are per kept row
    call_bytes = row_bytes_rw * T + T_src + 4.0 * T + 8.0 * (n_src + 1)   # + mask read, index written, cu in / out
    out = {
        "metric": METRIC, "value": T * args.steps / dt, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "ms_per_step_median": per_step[len(per_step) // 2] if per_step else None,
        "ms_per_step_min": per_step[0] if per_step else None,
        "config": {"workload": descr,
                   "hidden": H, "q_heads": shp["n_q_heads"], "kv_heads": shp["n_kv_heads"],
                   "head_dim": shp["head_dim"], "ffn": F, "tokens": T, "seq_len": S},
        "ms_per_step_untraced": ms_untraced,
        "step_tflops": (gemm_flops_step + attn_flops) / 1e12,
        "step_mfma_frac": (gemm_flops_step + attn_flops) / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "backward_only_ms": bwd_ms,
        "backward_only_mfma_frac": (gemm_flops_step + attn_flops) / (bwd_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "attention_backward": {"ms": attn_ms,
                               "tflops_5_contractions": attn_flops / 1e12,
                               "mfma_frac_5_contractions": attn_flops / max(attn_ms, 1e-9) / 1e9 / PEAK_BF16_TFLOPS,
                               "tflops_4_contractions": 0.8 * attn_flops / 1e12,
                               "mfma_frac_4_contractions": 0.8 * attn_flops / max(attn_ms, 1e-9) / 1e9 / PEAK_BF16_TFLOPS,
                               "note": "causal pairs only; 5 = S recompute, dP, dV, dK, dQ; 4 leaves the S recompute out; "
                                       "the two kernels execute 7 (S and dP are formed in both)"},
        "capture_gbps": pack_gbps,
        "capture_call_gbps": call_bytes / max(pack_ms, 1e-9) / 1e6,
        "capture_mask": "whole sequences (%d of %d prompts): a record feeds the backward only if every token of a kept "
                        "sequence is kept; the per-token Bernoulli(0.25) mask of config 3 is measured in also.config3" % (n_keep, n_src),
        "roofline": {"kernel": "k_gemm_mfma (all contractions of the layer backward)", "bound": "mfma",
                     "achieved": achieved_tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved_tf / PEAK_BF16_TFLOPS,
                     "traffic": load_traffic(args.traffic_json, "gemm_mfma_%s_bytes_per_launch" % args.workload),
                     "launches_per_step": gm[3] / args.steps, "avg_launch_ms": gm[2] / max(gm[3], 1)},
        "roofline_pack": {"kernel": "k_pack_gather", "bound": "hbm", "achieved": pack_gbps, "peak": PEAK_HBM_GBPS,
                          "unit": "GB/s", "frac": pack_gbps / PEAK_HBM_GBPS,
                          "traffic": load_traffic(args.traffic_json, "pack_gather_%s_bytes_per_launch" % args.workload),
                          "avg_launch_ms": pk[2] / max(pk[3], 1)},
        "kernel_ms_per_step": kms,
    }
    if "lora" in by:
        lo = by["lora"]
        out["roofline_lora"] = {"kernel": "k_lora_down / k_lora_up_* (rank-r adapter products)", "bound": "hbm",
                                "achieved": lo[1] / (lo[2] * 1e-3) / 1e9, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                "frac": lo[1] / (lo[2] * 1e-3) / 1e9 / PEAK_HBM_GBPS, "traffic": None,
                                "launches_per_step": lo[3] / args.steps}
    return out


def run_config4(args, torch, A):
    """32-layer 8B-shaped stack, 8 x 4096 tokens, vocab 128256: loss + backward from reused records
    (Section 1 of the paper) against forward recompute + the same backward (its separate-cluster baseline)."""
    import synth_inputs as synth
    dev, bf = "cuda", torch.bfloat16
    shp = synth.shape_dict("llama8b")
    shape = A.make_shape(*[shp[k] for k in synth.SHAPE_FIELDS], "bf16")
    H, QD, KD, F = shp["hidden"], shp["n_q_heads"] * shp["head_dim"], shp["n_kv_heads"] * shp["head_dim"], shp["ffn"]
    L, B, S, V = args.layers, 8, 4096, 128256
    T = B * S
    g = torch.Generator(device=dev).manual_seed(0)
    rnd = lambda shape_, std: (torch.randn(shape_, generator=g, device=dev, dtype=torch.float32) * std).to(bf)
    Ws = [{"Wq": rnd((QD, H), 0.02), "Wk": rnd((KD, H), 0.02), "Wv": rnd((KD, H), 0.02), "Wo": rnd((H, QD), 0.02),
           "Wg": rnd((F, H), 0.02), "Wu": rnd((F, H), 0.02), "Wd": rnd((H, F), 0.02),
           "g1": torch.ones(H, device=dev, dtype=bf), "g2": torch.ones(H, device=dev, dtype=bf)} for _ in range(L)]
    W_lm, g_final = rnd((V, H), 0.02), torch.ones(H, device=dev, dtype=bf)
    ids = torch.randint(0, V, (T,), generator=g, device=dev)
    emb = rnd((V, H), 0.02)
    X0 = emb[ids]
    del emb
    labels = torch.full((T,), -1, dtype=torch.int32, device=dev)
    lab2 = labels.view(B, S)
    lab2[:, :-1] = ids.view(B, S)[:, 1:].to(torch.int32)
    batch = A.Batch(synth.uniform_cu(B, S))
    ws_fwd = torch.empty(A.lib().alch_layer_forward_workspace_bytes(__import__("ctypes").byref(shape), T, S),
                         dtype=torch.uint8, device=dev)

    def forward():
        X, recs = X0, []
        for l in range(L):
            X, rec = A.alch_layer_forward(shape, batch, X, Ws[l], workspace=ws_fwd)
            recs.append(rec)
        return X, recs

    X_final, recs = forward()          # the records a serving prefill would have left behind
    r = args.lora_rank
    wflops = 2.0 if args.frozen_base else 4.0   # GEMM flops per parameter and token
    mode = "full backward"
    loss_mask = None
    if args.loss_mask:
        loss_mask = torch.from_numpy(synth.keep_mask(T, 0.25, 7)).to(dev)
    if r:
        # the paper's training setting (Section 6): rank-r adapters, here on all seven projections of every
        # layer; B = 0, the usual initialisation, so the records of the plain forward above are the adapted
        # model's records.  Base and head are frozen with --frozen-base, trained too without it.
        import ctypes
        dims = dict(q=(QD, H), k=(KD, H), v=(KD, H), o=(H, QD), g=(F, H), u=(F, H), d=(H, F))
        loras = [{p: (rnd((r, i), 0.05), torch.zeros((o, r), device=dev, dtype=bf)) for p, (o, i) in dims.items()}
                 for _ in range(L)]
        lgrads = [{"d" + m + p: torch.empty_like(ab[0] if m == "A" else ab[1]) for p, ab in lo.items() for m in "AB"}
                  for lo in loras]
        need = A.lib().alch_stack_backward_lora_workspace_bytes(ctypes.byref(shape), L, V, T, S, r)
        ws = torch.empty(need, dtype=torch.uint8, device=dev)
        bgrads = [({} if args.frozen_base else {"d" + k: torch.empty_like(v) for k, v in W.items()}) for W in Ws]
        mode = "rank-%d adapter gradients on a %s base" % (r, "frozen" if args.frozen_base else "trained")

        def backward(xf, rs, hooks=None):
            return A.alch_stack_backward_lora(shape, batch, rs, Ws, loras, r, 2.0, xf, g_final, W_lm, labels,
                                              loss_mask=loss_mask, grads_layers=bgrads, want_head=not args.frozen_base,
                                              lora_grads_layers=lgrads, hooks=hooks, workspace=ws)
    else:
        grads = [({} if args.frozen_base else {"d" + k: torch.empty_like(v) for k, v in W.items()}) for W in Ws]
        ws = torch.empty(A.stack_backward_workspace_bytes(shape, L, V, T, S), dtype=torch.uint8, device=dev)
        if args.frozen_base:
            mode = "data gradients only (frozen base and head)"

        def backward(xf, rs, hooks=None):
            return A.alch_stack_backward(shape, batch, rs, Ws, xf, g_final, W_lm, labels, loss_mask=loss_mask,
                                         grads_layers=grads, want_head=not args.frozen_base, hooks=hooks, workspace=ws)

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            out = fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps, out

    offload = None
    if args.six_stream or args.four_stream:
        # Section 4.3.2, per tensor: what is cheap to recompute is not kept (and, with --offload, not transferred)
        keep = ("X", "Q", "K", "V", "G", "U") if args.six_stream else ("X", "Q", "K", "V")
        recs = [{k: rec[k] for k in keep} for rec in recs]
        torch.cuda.empty_cache()
        mode += ", records hold %s only (the rest is recomputed by the backward)" % ", ".join(keep)
    if args.loss_mask:
        mode += ", loss on a Bernoulli(0.25) subset of the tokens (head and top layer run on the counted rows)"
    if args.offload:
        # Section 4.3: the records wait in pinned host memory; the walk prefetches them one layer ahead
        store = A.RecordStore(L, recs[0])
        for l in range(L):
            store.offload(l, recs[l])
        torch.cuda.synchronize()
        recs = None
        torch.cuda.empty_cache()
        t_reuse, out = timed(lambda: store.prefetching_backward(lambda saved, hooks: backward(X_final, saved, hooks)),
                             args.steps, args.warmup)
        offload = {"record_bytes_per_layer": store.bytes_per_layer,
                   "host_to_device_gbps": store.bytes_per_layer * L / t_reuse / 1e9}
        mode += ", records prefetched from pinned host memory"
    A.alch_trace_enable(True)
    if not args.offload:
        t_reuse, out = timed(lambda: backward(X_final, recs), args.steps, args.warmup)
    else:
        store.prefetching_backward(lambda saved, hooks: backward(X_final, saved, hooks))
        torch.cuda.synchronize()
    A.alch_trace_enable(False)
    trace = A.alch_trace_collect()
    loss = float(out["loss"].item())
    del recs

    def recompute_step():
        xf, rs = forward()
        return backward(xf, rs)
    t_rec, _ = timed(recompute_step, max(1, args.steps // 2), 1)
    n_traced_steps = 1 if args.offload else args.steps + args.warmup

    gm = [r for r in trace if r[0] == "gemm_mfma"]
    gm_ms = sum(r[3] for r in gm)
    achieved_tf = sum(r[1] for r in gm) / (gm_ms * 1e-3) / 1e12
    P = 2 * H * QD + 2 * H * KD + 3 * H * F
    head_flops = (4.0 if args.frozen_base else 6.0) * V * H   # logits + dHf (+ dW_lm)
    gemm_flops = T * (L * wflops * P + head_flops)
    if args.loss_mask:
        # the head and the row-local products of the top layer run on the counted rows only (their launches are
        # traced without flops because the row count lives on the device): count what the method must touch
        n_cnt = int(((labels >= 0) & (loss_mask != 0)).sum().item())
        p_rows = 3 * H * F + H * QD
        gemm_flops = T * wflops * ((L - 1) * P + (P - p_rows)) + n_cnt * (wflops * p_rows + head_flops)
        achieved_tf = gemm_flops / (gm_ms / n_traced_steps * 1e-3) / 1e12
    flops = gemm_flops + L * 10.0 * shp["head_dim"] * shp["n_q_heads"] * B * S * (S + 1) / 2
    by = {}
    for kind, fl, nb, ms in trace:
        by[kind] = by.get(kind, 0.0) + ms
    n_traced = n_traced_steps
    res = {
        "metric": METRIC, "value": T / t_reuse, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": t_reuse * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config4: %d-layer Llama-3-8B-shaped stack, bf16, 8 x 4096 tokens, vocab 128256, "
                               "cross-entropy + %s from reused records" % (L, mode),
                   "layers": L, "tokens": T, "seq_len": S, "vocab": V},
        "loss": loss, "loss_expected_random_init": float(np.log(V) + 0.5 * 0.02 ** 2 * H),
        "step_tflops": flops / 1e12, "step_mfma_frac": flops / t_reuse / 1e12 / PEAK_BF16_TFLOPS,
        "recompute_tokens_per_s": T / t_rec, "reuse_speedup_over_recompute": t_rec / t_reuse,
        "roofline": {"kernel": "k_gemm_mfma (all contractions of the stack backward)", "bound": "mfma",
                     "achieved": achieved_tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved_tf / PEAK_BF16_TFLOPS, "traffic": None,
                     "launches_per_step": len(gm) / n_traced, "avg_launch_ms": gm_ms / max(len(gm), 1)},
        "kernel_ms_per_step": {k: v / n_traced for k, v in by.items()},
    }
    if offload:
        res["offload"] = offload
    return res


def run_dpo(args, torch, A):
    """Preference alignment on shared prefills (Section 4.1, Section 6 of the paper): 8 prompts x 2048 tokens whose
    records a serving prefill left behind, each with a chosen and a rejected response of 128 tokens.  A step =
    forward of the response tokens alone on the prompts' saved K/V (every layer) + DPO loss + backward through
    prompts and responses.  Compared with the path without reuse: prefill of prompt + response twice
    (16 sequences x 2176 tokens), the same loss, the same backward."""
    import ctypes
    import synth_inputs as synth
    dev, bf = "cuda", torch.bfloat16
    shp = synth.shape_dict("llama8b")
    shape = A.make_shape(*[shp[k] for k in synth.SHAPE_FIELDS], "bf16")
    H, QD, KD, F = shp["hidden"], shp["n_q_heads"] * shp["head_dim"], shp["n_kv_heads"] * shp["head_dim"], shp["ffn"]
    L, NP, P, R, V, beta = args.layers, 8, 2048, 128, 128256, 0.1
    b = synth.preference_batch([P] * NP, [[R, R]] * NP, V, 0)
    T, Tp = int(b["cu"][-1]), NP * P
    g = torch.Generator(device=dev).manual_seed(0)
    rnd = lambda shape_, std: (torch.randn(shape_, generator=g, device=dev, dtype=torch.float32) * std).to(bf)
    Ws = [{"Wq": rnd((QD, H), 0.02), "Wk": rnd((KD, H), 0.02), "Wv": rnd((KD, H), 0.02), "Wo": rnd((H, QD), 0.02),
           "Wg": rnd((F, H), 0.02), "Wu": rnd((F, H), 0.02), "Wd": rnd((H, F), 0.02),
           "g1": torch.ones(H, device=dev, dtype=bf), "g2": torch.ones(H, device=dev, dtype=bf)} for _ in range(L)]
    W_lm, g_final = rnd((V, H), 0.02), torch.ones(H, device=dev, dtype=bf)
    emb = rnd((V, H), 0.02)
    X0 = emb[torch.from_numpy(b["tokens"]).to(dev).long()]
    del emb
    ref = torch.full((2 * NP,), -float(R) * float(np.log(V)), dtype=torch.float32, device=dev)  # a uniform reference model
    r = args.lora_rank
    frozen = args.frozen_base
    loras = None
    if r:
        dims = dict(q=(QD, H), k=(KD, H), v=(KD, H), o=(H, QD), g=(F, H), u=(F, H), d=(H, F))
        loras = [{p: (rnd((r, i), 0.05), torch.zeros((o, r), device=dev, dtype=bf)) for p, (o, i) in dims.items()}
                 for _ in range(L)]
    want = () if frozen else A.WEIGHT_KEYS
    grads = [({} if frozen else {"d" + k: torch.empty_like(v) for k, v in W.items()}) for W in Ws]
    lgrads = None if not r else [{"d" + m + p: torch.empty_like(ab[0] if m == "A" else ab[1]) for p, ab in lo.items()
                                  for m in "AB"} for lo in loras]
    if r:
        need = A.lib().alch_stack_backward_lora_workspace_bytes(ctypes.byref(shape), L, V, 16 * (P + R), P + R, r)
    else:
        need = A.stack_backward_workspace_bytes(shape, L, V, 16 * (P + R), P + R)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    ws_fwd = torch.empty(A.lib().alch_layer_forward_workspace_bytes(ctypes.byref(shape), 16 * (P + R), P + R),
                         dtype=torch.uint8, device=dev)

    def backward(batch, recs, xf, items):
        return A.alch_stack_backward_dpo(shape, batch, recs, Ws, xf, g_final, W_lm, items[0], items[1], items[2], ref, beta,
                                         lora_layers=loras, rank=r, scale=2.0, want=want, want_head=not frozen,
                                         lora_grads_layers=lgrads, grads_layers=grads, workspace=ws)

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            out = fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps, out

    # ---- reuse: the prompts' rows of every record exist (written once, untimed: the serving prefill) ----
    batch = A.Batch(b["cu"], positions=b["positions"], prefix=b["prefix"])
    prompts_only = A.Batch(b["cu"][:NP + 1])
    acts, recs = [X0], []
    widths = dict(X=H, X2=H, Q=QD, K=KD, V=KD, O=QD, G=F, U=F)
    for l in range(L):
        rec = {k: torch.empty((T, w), dtype=bf, device=dev) for k, w in widths.items() if k != "X"}
        rec["X"] = acts[l]
        rec["LSE"] = torch.empty((T, shp["n_q_heads"]), dtype=torch.float32, device=dev)
        Y = torch.empty((T, H), dtype=bf, device=dev)
        A.alch_layer_forward(shape, prompts_only, acts[l], Ws[l], workspace=ws_fwd, rec=rec, Y=Y)   # rows of the prompts
        recs.append(rec)
        acts.append(Y)
    items = (b["item_row"], b["item_label"], b["item_slot"])

    def reuse_step():
        for l in range(L):   # the responses alone, on the prompts' saved keys and values
            A.alch_layer_forward(shape, batch, acts[l], Ws[l], workspace=ws_fwd, seq_begin=NP, rec=recs[l], Y=acts[l + 1])
        return backward(batch, recs, acts[L], items)

    A.alch_trace_enable(True)
    t_reuse, out = timed(reuse_step, args.steps, args.warmup)
    A.alch_trace_enable(False)
    trace = A.alch_trace_collect()
    loss = float(out["loss"].item())
    rec_bytes = sum(t.numel() * t.element_size() for rec in recs for t in rec.values())
    del recs, acts
    torch.cuda.empty_cache()

    # ---- no reuse: prompt + response prefilled once per response ----
    cu_d = synth.uniform_cu(2 * NP, P + R)
    src = np.concatenate([np.concatenate([np.arange(g_ * P, (g_ + 1) * P), np.arange(Tp + k * R, Tp + (k + 1) * R)])
                          for g_ in range(NP) for k in (2 * g_, 2 * g_ + 1)])
    X0d = X0[torch.from_numpy(src).to(dev)]
    Td = int(cu_d[-1])
    rows, labels, slots = [], [], []
    tok = b["tokens"]
    for k in range(2 * NP):
        a = k * (P + R)
        rows += list(range(a + P - 1, a + P + R - 1))
        labels += list(tok[Tp + k * R: Tp + (k + 1) * R])
        slots += [k] * R
    items_d = (np.asarray(rows, np.int32), np.asarray(labels, np.int32), np.asarray(slots, np.int32))
    batch_d = A.Batch(cu_d)

    def dup_step():
        X, rs = X0d, []
        for l in range(L):
            X, rec = A.alch_layer_forward(shape, batch_d, X, Ws[l], workspace=ws_fwd)
            rs.append(rec)
        return backward(batch_d, rs, X, items_d), rs

    t_dup, (out_d, rs) = timed(dup_step, max(1, args.steps // 2), 1)
    loss_d = float(out_d["loss"].item())
    rec_bytes_d = sum(t.numel() * t.element_size() for rec in rs for t in rec.values())
    del rs

    gm = [x for x in trace if x[0] == "gemm_mfma"]
    gm_ms = sum(x[3] for x in gm)
    achieved_tf = sum(x[1] for x in gm) / (gm_ms * 1e-3) / 1e12
    n_traced = args.steps + args.warmup
    by = {}
    for kind, fl, nb, ms in trace:
        by[kind] = by.get(kind, 0.0) + ms
    mode = ("rank-%d adapters on a %s base" % (r, "frozen" if frozen else "trained")) if r else \
           ("data gradients only (frozen base and head)" if frozen else "full weight gradients")
    return {
        "metric": METRIC, "value": T / t_reuse, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": t_reuse * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "dpo: %d-layer Llama-3-8B-shaped stack, bf16, %d prompts x %d tokens (records reused) + "
                               "chosen and rejected response of %d tokens each on the shared prompt K/V, vocab %d, DPO "
                               "loss, %s" % (L, NP, P, R, V, mode),
                   "layers": L, "tokens": T, "prompt_len": P, "response_len": R, "vocab": V},
        "loss": loss, "loss_without_reuse": loss_d,
        "without_reuse_ms_per_step": t_dup * 1e3, "without_reuse_tokens_per_s": T / t_dup,
        "reuse_speedup": t_dup / t_reuse,
        "record_bytes_shared_prompt": rec_bytes, "record_bytes_without_reuse": rec_bytes_d,
        "record_memory_saving": 1.0 - rec_bytes / rec_bytes_d,
        "roofline": {"kernel": "k_gemm_mfma (all contractions of the response forward and the backward)", "bound": "mfma",
                     "achieved": achieved_tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved_tf / PEAK_BF16_TFLOPS, "traffic": None,
                     "launches_per_step": len(gm) / n_traced, "avg_launch_ms": gm_ms / max(len(gm), 1)},
        "kernel_ms_per_step": {k: v / n_traced for k, v in by.items()},
    }


def run_config3(args, torch, A):
    import synth_inputs as synth
    dev = "cuda"
    n_layers, n_prompts = 32, 32
    lens = synth.random_lengths(n_prompts, 256, 4096, 0)
    cu = synth.ragged_cu(lens)
    T = int(cu[-1])
    mask_np = synth.keep_mask(T, 0.25, 1)
    n_kept = int(mask_np.sum())
    mask = torch.from_numpy(mask_np).to(dev)
    batch = A.Batch(cu)
    # two rotating sets of source buffers so that no layer call finds its source in cache
    sets = []
    for i in range(2):
        hid = torch.empty((T, 4096), dtype=torch.bfloat16, device=dev).normal_()
        qkv = torch.empty((T, 6144), dtype=torch.bfloat16, device=dev).normal_()
        gu = torch.empty((T, 28672), dtype=torch.bfloat16, device=dev).normal_()
        sets.append([hid, qkv[:, :4096], qkv[:, 4096:5120], qkv[:, 5120:], gu[:, :14336], gu[:, 14336:]])
    cap = n_kept
    dsts = [[torch.empty((cap, s.shape[1]), dtype=s.dtype, device=dev) for s in sets[0]] for _ in range(2)]
    ws = torch.empty(A.lib().alch_capture_pack_workspace_bytes(T), dtype=torch.uint8, device=dev)

    def step():
        for l in range(n_layers):
            if l == 0 or not args.scan_once:
                kept, _, status, _ = A.alch_capture_pack(batch, mask, sets[l & 1], capacity=cap, dsts=dsts[l & 1], workspace=ws)
            else:   # the mask of a prefill batch is the same for every layer: its index is reused
                A.alch_capture_gather(batch, kept, status, sets[l & 1], capacity=cap, dsts=dsts[l & 1])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    A.alch_trace_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    A.alch_trace_enable(False)
    trace = A.alch_trace_collect()
    pk = [r for r in trace if r[0] == "pack_gather"]
    ms = sum(r[3] for r in pk)
    row_rw = pk[0][2]
    gbps = row_rw * n_kept * len(pk) / (ms * 1e-3) / 1e9
    scans = 1 if args.scan_once else n_layers
    total_bytes = row_rw * n_kept * n_layers + (T + 4 * n_kept + 8 * (n_prompts + 1)) * scans
    return {
        "metric": METRIC, "value": total_bytes * args.steps / dt / 1e9, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "config3: capture/pack only, 32 layers x 32 prompts (lengths U[256,4096]), keep ~ "
                               "Bernoulli(0.25), 6 bf16 streams per layer from fused qkv / gate-up buffers" +
                               (", mask scanned once per batch" if args.scan_once else ""),
                   "tokens": T, "kept": n_kept, "bytes_per_kept_token_per_layer": row_rw / 2},
        "capture_gbps": gbps,
        "capture_call_gbps": total_bytes * args.steps / ((ms + sum(r[3] for r in trace if r[0] == "pack_scan")) * 1e-3) / 1e9,
        "roofline": {"kernel": "k_pack_gather", "bound": "hbm", "achieved": gbps, "peak": PEAK_HBM_GBPS,
                     "unit": "GB/s", "frac": gbps / PEAK_HBM_GBPS,
                     "traffic": load_traffic(args.traffic_json, "pack_gather_config3_bytes_per_launch"),
                     "algorithmic_bytes_per_launch": row_rw * n_kept,
                     "avg_launch_ms": ms / len(pk)},
        "whole_job_frac_of_hbm_peak": total_bytes * args.steps / dt / 1e9 / PEAK_HBM_GBPS,
    }


def run_copy(args, torch, A):
    """Calibration workload for the HBM byte counters: a plain device-to-device copy of known size."""
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(args.warmup):
        dst.copy_(src)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        dst.copy_(src)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    gbps = 2.0 * n * args.steps / dt / 1e9
    return {"metric": "plain copy GB/s (counter calibration)", "value": gbps, "unit": "GB/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
            "config": {"workload": "copy: 1 GiB read + 1 GiB written per step", "bytes_read": n, "bytes_written": n},
            "roofline": {"kernel": "device copy", "bound": "hbm", "achieved": gbps, "peak": PEAK_HBM_GBPS,
                         "unit": "GB/s", "frac": gbps / PEAK_HBM_GBPS, "traffic": None}}


def run_gemm(args, torch, A):
    """Ceiling check of the contraction kernel: every product shape of the config-2 layer backward (and a square
    one), timed through alch_gemm and through torch.matmul (the vendor library) on the same operands, with
    Gaussian and with all-zero data (the matrix pipes draw less power on zeros, which shows how far the clock
    granted under load, not the kernel, sets the rate)."""
    dev, bf = "cuda", torch.bfloat16
    T, H, F, QKV = 8192, 4096, 14336, 6144
    shapes = [("dAct = dY Wd", T, F, H, True, False), ("dH2 = dGU [Wg;Wu]", T, H, 2 * F, True, False),
              ("dO = dX2 Wo", T, H, H, True, False), ("dH1 = dQKV Wqkv", T, H, QKV, True, False),
              ("dWd = dY^T Act", H, F, T, False, False), ("dWgu = dGU^T H2", 2 * F, H, T, False, False),
              ("dWo = dX2^T O", H, H, T, False, False), ("dWqkv = dQKV^T H1", QKV, H, T, False, False),
              ("square, y = x W^T", 8192, 8192, 8192, True, True)]
    ws = torch.empty(A.lib().alch_gemm_workspace_bytes(), dtype=torch.uint8, device=dev)
    g = torch.Generator(device=dev).manual_seed(0)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    rows, tot = [], {"alch": 0.0, "vendor": 0.0, "flops": 0.0}
    for name, M, N, K, a_k, b_k in shapes:
        row = {"product": name, "M": M, "N": N, "K": K}
        for data in ("gaussian", "zeros"):
            mk = (lambda *sh: torch.randn(sh, generator=g, device=dev, dtype=torch.float32).to(bf)) if data == "gaussian" \
                else (lambda *sh: torch.zeros(sh, device=dev, dtype=bf))
            a = mk(M, K) if a_k else mk(K, M)
            b = mk(N, K) if b_k else mk(K, N)
            out = torch.empty((M, N), dtype=bf, device=dev)
            am = a if a_k else a.t()
            bm = b.t() if b_k else b
            ms_a = timed(lambda: A.alch_gemm(M, N, [(a, b, K)], a_k, b_k, out=out, workspace=ws))
            ms_v = timed(lambda: torch.matmul(am, bm, out=out))
            fl = 2.0 * M * N * K
            row[data] = {"alch_tflops": fl / ms_a / 1e9, "vendor_tflops": fl / ms_v / 1e9}
            if data == "gaussian" and not name.startswith("square"):
                tot["alch"] += ms_a; tot["vendor"] += ms_v; tot["flops"] += fl
            del a, b, out
        rows.append(row)
    ach = tot["flops"] / tot["alch"] / 1e9
    return {"metric": "contraction TFLOP/s over the config-2 products (ceiling check against the vendor library)",
            "value": ach, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": tot["alch"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "gemm: the eight products of the config-2 layer backward, one launch each, Gaussian data"},
            "vendor_tflops": tot["flops"] / tot["vendor"] / 1e9, "products": rows,
            "roofline": {"kernel": "k_gemm_mfma", "bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS,
                         "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": None}}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); sharding over several GPUs (by sequence, one "
              "exchange of the weight gradients) is described in the design notes and not built", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2503_01066_amd as A
    A.lib()  # fails loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    runners = {"config2": run_layer, "config5": run_layer, "short": run_layer, "config3": run_config3, "config4": run_config4,
               "dpo": run_dpo, "copy": run_copy, "gemm": run_gemm}
    out = runners[args.workload](args, torch, A)
    P_tok_cfg2 = 4.0 * (2 * 4096 * 4096 + 2 * 4096 * 1024 + 3 * 4096 * 14336) + 10.0 * 128 * 32 * 2049 / 2

    def config4_baseline(res, layer_baseline):
        # extrapolated, and labelled so: one layer on 4 x 2048 tokens, scaled by flops
        b = dict(layer_baseline)
        per_tok = res["step_tflops"] * 1e12 / res["config"]["tokens"]
        b["value"] = b["value"] * P_tok_cfg2 / per_tok
        b["sample"] = "EXTRAPOLATED by flop count from: " + b["sample"]
        return b

    if not args.no_cpu_baseline and args.workload == "config4":
        out["cpu_baseline"] = config4_baseline(out, cpu_baseline_layer("config2"))
    elif not args.no_cpu_baseline and args.workload == "dpo":
        out["cpu_baseline"] = cpu_baseline_dpo(args.layers)
    elif not args.no_cpu_baseline and args.workload not in ("copy", "gemm"):
        out["cpu_baseline"] = cpu_baseline_config3(layers=32 if args.cpu_baseline_full else 4) if args.workload == "config3" \
            else cpu_baseline_layer(args.workload, full=args.cpu_baseline_full)

    if args.workload == "config2" and not args.headline_only and not (args.lora_rank or args.frozen_base or args.loss_mask
                                                                        or args.six_stream or args.four_stream):
        # The other configurations of the method's evaluation, measured in the same run, each with its own step
        # count, roofline and oracle baseline.  A failure in one of them is recorded and does not hide the headline.
        import copy
        import gc
        keep = ("value", "unit", "steps", "warmup", "ms_per_step", "ms_per_step_untraced", "dtype", "config", "roofline",
                "roofline_pack", "capture_gbps", "capture_call_gbps", "whole_job_frac_of_hbm_peak", "step_tflops",
                "step_mfma_frac", "backward_only_ms", "backward_only_mfma_frac", "attention_backward", "kernel_ms_per_step",
                "loss", "loss_expected_random_init", "recompute_tokens_per_s", "reuse_speedup_over_recompute", "cpu_baseline")
        also = {}

        def leg(name, workload, steps, warmup, baseline, **flags):
            a = copy.copy(args)
            a.workload, a.steps, a.warmup = workload, steps, warmup
            for k, v in flags.items():
                setattr(a, k, v)
            try:
                gc.collect()
                torch.cuda.empty_cache()
                res = runners[workload](a, torch, A)
                if baseline is not None and not args.no_cpu_baseline:
                    res["cpu_baseline"] = baseline(res)
                also[name] = {k: res[k] for k in keep if k in res}
            except Exception as e:   # noqa: BLE001  (reported in the line, never silently dropped)
                also[name] = {"error": "%s: %s" % (type(e).__name__, e)}

        leg("config3", "config3", 10, 3, lambda r: cpu_baseline_config3(layers=32))
        base5 = {}
        leg("config5_dense", "config5", 10, 2, lambda r: base5.setdefault("b", cpu_baseline_layer("config5", full=True)))
        leg("config5_loss_mask", "config5", 10, 2, lambda r: base5.get("b") or cpu_baseline_layer("config5", full=True), loss_mask=True)
        leg("config4", "config4", 2, 1, lambda r: config4_baseline(r, out["cpu_baseline"]) if "cpu_baseline" in out else None)
        out["also"] = also
    print(json.dumps(out))


if __name__ == "__main__":
    main()
