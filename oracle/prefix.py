"""Oracle for sequences that share a prefix, and for the DPO loss on them.

Test infrastructure only (see the package docstring).  All arithmetic is float64.

Paper basis: Section 4.1, preference alignment: only the prefill of the prompt is recorded (its
activations and its KV cache); the loss is computed by running the response tokens alone, which attend
to the saved KV cache of the prompt; the chosen and the rejected response share one prompt, so both
forward passes share that KV cache and the activations that belong to it.  Section 6, "Training": DPO is
the example loss; the rejected response is the model's own output and the chosen one has the same length.
Section 4.3.2 repeats that the prompt is prefilled once for all forward passes over it.

The paper prints no formula for this case.  Readings taken here:
  * a batch is a list of sequences (cu_seqlens) plus `prefix[s]`: -1, or the index of an earlier sequence
    that has no prefix itself (a prompt).  Token i of sequence s attends to every token of the prefix
    sequence and to tokens j <= i of its own sequence; its rotary position is len(prefix) + i.  A prompt
    attends causally to itself only, exactly as in the plain layer.  Nothing else of the layer changes:
    every other step is row-local.
  * one backward pass covers prompts and responses together.  The keys and values of a prompt receive
    gradient from its own tokens and from every response that attends to them, so the prompt rows of the
    layer input receive gradient although they carry no loss term (Section 4.1: the activations of the
    prompt are saved so that the training step can go through them).
  * DPO (Rafailov et al. 2023), for pair p with chosen response c and rejected response r:
        z_p = beta * [(pi_c - ref_c) - (pi_r - ref_r)],   loss = mean_p -log sigmoid(z_p),
    pi_s = sum of log-probabilities of the scored tokens of s under the model, ref_s the same number under
    the frozen reference model (an input).  A scored token is an `item` (row, label, slot): the
    log-probability of `label` is read from the LM-head row computed from stack-output row `row`, and adds
    to slot 2p (chosen) or 2p+1 (rejected).  The first token of a response is predicted by the last prompt
    row, so that row appears in two items, one per response, with different labels.
"""
import numpy as np

from .layer import (RECORD_KEYS, _rms_norm, _rms_norm_backward, _rope, _sigmoid)


def visibility(cu_seqlens, prefix):
    """allowed[i, j]: token i (row of the batch) attends to token j."""
    T = int(cu_seqlens[-1])
    allowed = np.zeros((T, T), dtype=bool)
    for s in range(len(cu_seqlens) - 1):
        a, b = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        allowed[a:b, a:b] = np.tril(np.ones((b - a, b - a), dtype=bool))
        p = int(prefix[s]) if prefix is not None else -1
        if p >= 0:
            assert p < s and int(prefix[p]) < 0, "a prefix is an earlier sequence without a prefix of its own"
            allowed[a:b, int(cu_seqlens[p]):int(cu_seqlens[p + 1])] = True
    return allowed


def prefix_positions(cu_seqlens, prefix):
    """Rotary position of every row: index inside the sequence plus the length of its prefix."""
    T = int(cu_seqlens[-1])
    pos = np.zeros(T, dtype=np.float64)
    for s in range(len(cu_seqlens) - 1):
        a, b = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        p = int(prefix[s]) if prefix is not None else -1
        base = int(cu_seqlens[p + 1]) - int(cu_seqlens[p]) if p >= 0 else 0
        pos[a:b] = base + np.arange(b - a)
    return pos


def _attention(shape, allowed, Q, K, V):
    """Masked grouped-query attention over the whole batch.  Returns (O [T,Hq,D], LSE [T,Hq])."""
    T = Q.shape[0]
    Hq, Hkv, D = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    G = Hq // Hkv
    O = np.zeros((T, Hq, D), dtype=np.float64)
    LSE = np.zeros((T, Hq), dtype=np.float64)
    for h in range(Hq):
        sc = np.where(allowed, Q[:, h] @ K[:, h // G].T / np.sqrt(D), -np.inf)
        m = sc.max(axis=1, keepdims=True)
        e = np.exp(sc - m)
        l = e.sum(axis=1, keepdims=True)
        O[:, h] = (e / l) @ V[:, h // G]
        LSE[:, h] = (m + np.log(l))[:, 0]
    return O, LSE


def layer_forward_prefix(shape, cu_seqlens, prefix, X, W):
    """The decoder layer on a batch with shared prefixes.  Returns (Y, record)."""
    X = np.asarray(X, dtype=np.float64)
    T, H = X.shape
    Hq, Hkv, D = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    pos = prefix_positions(cu_seqlens, prefix)
    H1, _ = _rms_norm(X, W["g1"], shape.rms_eps)
    Q = _rope((H1 @ W["Wq"].T).reshape(T, Hq, D), pos, shape.rope_base, +1)
    K = _rope((H1 @ W["Wk"].T).reshape(T, Hkv, D), pos, shape.rope_base, +1)
    V = (H1 @ W["Wv"].T).reshape(T, Hkv, D)
    O, LSE = _attention(shape, visibility(cu_seqlens, prefix), Q, K, V)
    O = O.reshape(T, Hq * D)
    X2 = X + O @ W["Wo"].T
    H2, _ = _rms_norm(X2, W["g2"], shape.rms_eps)
    Gt = H2 @ W["Wg"].T
    U = H2 @ W["Wu"].T
    Y = X2 + (Gt * _sigmoid(Gt) * U) @ W["Wd"].T
    rec = dict(X=X, X2=X2, Q=Q.reshape(T, Hq * D), K=K.reshape(T, Hkv * D), V=V.reshape(T, Hkv * D),
               O=O, LSE=LSE, G=Gt, U=U)
    return Y, rec


def layer_backward_reuse_prefix(shape, cu_seqlens, prefix, rec, W, dY):
    """Backward of layer_forward_prefix from the saved record (consumed as given).
    Returns dict: dX and the nine weight / gain gradients."""
    X, X2, Q, K, V, O, LSE, Gt, U = (np.asarray(rec[k], dtype=np.float64) for k in RECORD_KEYS)
    T, H = X.shape
    Hq, Hkv, D = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    G = Hq // Hkv
    pos = prefix_positions(cu_seqlens, prefix)
    allowed = visibility(cu_seqlens, prefix)
    dY = np.asarray(dY, dtype=np.float64)

    sig = _sigmoid(Gt)
    Act = Gt * sig * U
    dAct = dY @ W["Wd"]
    dWd = dY.T @ Act
    dG = dAct * U * sig * (1.0 + Gt * (1.0 - sig))
    dU = dAct * Gt * sig
    dH2 = dG @ W["Wg"] + dU @ W["Wu"]
    H2, r2 = _rms_norm(X2, W["g2"], shape.rms_eps)
    dWg, dWu = dG.T @ H2, dU.T @ H2
    dX2n, dg2 = _rms_norm_backward(dH2, X2, W["g2"], r2)
    dX2 = dY + dX2n
    dO = (dX2 @ W["Wo"]).reshape(T, Hq, D)
    dWo = dX2.T @ O

    Qh, Kh, Vh, Oh = Q.reshape(T, Hq, D), K.reshape(T, Hkv, D), V.reshape(T, Hkv, D), O.reshape(T, Hq, D)
    delta = np.sum(dO * Oh, axis=-1)
    dQ, dK, dV = np.zeros_like(Qh), np.zeros_like(Kh), np.zeros_like(Vh)
    scale = 1.0 / np.sqrt(D)
    for h in range(Hq):
        kv = h // G
        P = np.where(allowed, np.exp(Qh[:, h] @ Kh[:, kv].T * scale - LSE[:, h][:, None]), 0.0)
        dV[:, kv] += P.T @ dO[:, h]
        dS = P * (dO[:, h] @ Vh[:, kv].T - delta[:, h][:, None])
        dQ[:, h] = dS @ Kh[:, kv] * scale
        dK[:, kv] += dS.T @ Qh[:, h] * scale

    dQp = _rope(dQ, pos, shape.rope_base, -1).reshape(T, Hq * D)
    dKp = _rope(dK, pos, shape.rope_base, -1).reshape(T, Hkv * D)
    dVp = dV.reshape(T, Hkv * D)
    dH1 = dQp @ W["Wq"] + dKp @ W["Wk"] + dVp @ W["Wv"]
    H1, r1 = _rms_norm(X, W["g1"], shape.rms_eps)
    dXn, dg1 = _rms_norm_backward(dH1, X, W["g1"], r1)
    return dict(dX=dX2 + dXn, dWq=dQp.T @ H1, dWk=dKp.T @ H1, dWv=dVp.T @ H1, dWo=dWo, dWg=dWg, dWu=dWu,
                dWd=dWd, dg1=dg1, dg2=dg2)


def stack_forward_prefix(shape, cu_seqlens, prefix, X0, layers_W):
    X = np.asarray(X0, dtype=np.float64)
    recs = []
    for W in layers_W:
        X, rec = layer_forward_prefix(shape, cu_seqlens, prefix, X, W)
        recs.append(rec)
    return X, recs


def dpo_head(shape, X_final, g_final, W_lm, item_row, item_label, item_slot, ref_logp, beta):
    """DPO loss over pairs and its gradients.  item_*: one entry per scored token; ref_logp [2 * n_pairs]
    (slot 2p chosen, 2p+1 rejected).  Returns (loss, dX_final, dg_final, dW_lm, z [n_pairs])."""
    X_final = np.asarray(X_final, dtype=np.float64)
    g_final = np.asarray(g_final, dtype=np.float64)
    W_lm = np.asarray(W_lm, dtype=np.float64)
    rows = np.asarray(item_row, dtype=np.int64)
    labels = np.asarray(item_label, dtype=np.int64)
    slots = np.asarray(item_slot, dtype=np.int64)
    ref = np.asarray(ref_logp, dtype=np.float64)
    n_pairs = ref.shape[0] // 2
    dX = np.zeros_like(X_final)
    if n_pairs == 0:
        return 0.0, dX, np.zeros_like(g_final), np.zeros_like(W_lm), np.zeros(0)
    Hf, rf = _rms_norm(X_final, g_final, shape.rms_eps)
    logits = Hf[rows] @ W_lm.T                                   # one LM-head row per item
    m = logits.max(axis=1, keepdims=True)
    logp = logits - (m + np.log(np.sum(np.exp(logits - m), axis=1, keepdims=True)))
    pi = np.zeros(2 * n_pairs)
    np.add.at(pi, slots, logp[np.arange(len(rows)), labels])
    z = beta * ((pi[0::2] - ref[0::2]) - (pi[1::2] - ref[1::2]))
    loss = float(np.mean(np.logaddexp(0.0, -z)))                  # -log sigmoid(z)
    # d loss / d z_p = -sigmoid(-z_p) / n_pairs;  d z_p / d pi = +beta (chosen), -beta (rejected)
    dz = -1.0 / (1.0 + np.exp(z)) / n_pairs
    dpi = np.zeros(2 * n_pairs)
    dpi[0::2], dpi[1::2] = beta * dz, -beta * dz
    w = dpi[slots]                                               # weight of each item's log-probability
    dlogits = -w[:, None] * np.exp(logp)                         # d logp[label] / d logits = onehot - softmax
    dlogits[np.arange(len(rows)), labels] += w
    dW_lm = dlogits.T @ Hf[rows]
    dHf = np.zeros_like(X_final)
    np.add.at(dHf, rows, dlogits @ W_lm)
    dX, dg_final = _rms_norm_backward(dHf, X_final, g_final, rf)
    return loss, dX, dg_final, dW_lm, z


def stack_backward_dpo(shape, cu_seqlens, prefix, recs, layers_W, X_final, g_final, W_lm, item_row, item_label,
                       item_slot, ref_logp, beta):
    """DPO head on the saved stack output, then the layers from the output layer to the input layer
    (Section 4.2), each from its own saved record.  Returns dict: loss, z, dX_embed, dg_final, dW_lm, layers."""
    loss, dX, dg_final, dW_lm, z = dpo_head(shape, X_final, g_final, W_lm, item_row, item_label, item_slot,
                                            ref_logp, beta)
    per_layer = [None] * len(layers_W)
    for l in range(len(layers_W) - 1, -1, -1):
        g = layer_backward_reuse_prefix(shape, cu_seqlens, prefix, recs[l], layers_W[l], dX)
        dX = g["dX"]
        per_layer[l] = g
    return dict(loss=loss, z=z, dX_embed=dX, dg_final=dg_final, dW_lm=dW_lm, layers=per_layer)


def stack_backward_dpo_lora(shape, cu_seqlens, prefix, recs, layers_W, layers_lora, scale, X_final, g_final, W_lm,
                            item_row, item_label, item_slot, ref_logp, beta):
    """stack_backward_dpo for layers that carry low-rank adapters (Section 6: the evaluated models carry a
    rank-8 adapter).  Same definition as the adapter oracle of the plain layer: the adapted projection is the
    plain one at W' = W + scale * B A, so dA = scale * B^T dW', dB = scale * dW' A^T with dW' the weight
    gradient of the shared-prefix layer at W'.  The head carries no adapter."""
    from .lora import merged_weights
    loss, dX, dg_final, dW_lm, z = dpo_head(shape, X_final, g_final, W_lm, item_row, item_label, item_slot,
                                            ref_logp, beta)
    per_layer = [None] * len(layers_W)
    for l in range(len(layers_W) - 1, -1, -1):
        g = layer_backward_reuse_prefix(shape, cu_seqlens, prefix, recs[l], merged_weights(layers_W[l], layers_lora[l], scale), dX)
        for p, (A, B) in layers_lora[l].items():
            dWm = g["dW" + p]
            g["dA" + p] = scale * np.asarray(B, dtype=np.float64).T @ dWm
            g["dB" + p] = scale * dWm @ np.asarray(A, dtype=np.float64).T
        dX = g["dX"]
        per_layer[l] = g
    return dict(loss=loss, z=z, dX_embed=dX, dg_final=dg_final, dW_lm=dW_lm, layers=per_layer)
