"""Oracle for the decoder layer with low-rank adapters (LoRA) on its projections.

Test infrastructure only (see the package docstring).  All arithmetic is float64.

Paper basis: Section 3, assumption A1 (training on the serving system is parameter
efficient fine-tuning such as LoRA: the base model stays frozen and only small
low-rank adapters are updated) and Section 6, "Training" (the evaluated models carry
a LoRA adapter of rank 8).  The paper does not say which projections carry the
adapter nor how it is scaled; readings taken here:
  * any of the seven projections p in (q, k, v, o, g, u, d) may carry an adapter
    (A_p [r, in_p], B_p [out_p, r]); a projection without one is absent from `lora`;
  * the adapted projection is y = x W_p^T + scale * (x A_p^T) B_p^T, one `scale`
    (alpha / r of the LoRA paper) for the whole layer;
  * the saved record is the one the serving forward produced with the adapters
    attached, i.e. Q, K, V, O, G, U already contain the low-rank terms.

Definition used for the backward: the adapted projection is the plain projection
with the weight W'_p = W_p + scale * B_p A_p.  W'_p depends on (W_p, A_p, B_p)
linearly in each, so by the chain rule
    dX      = input gradient of the plain layer with weights W',
    dW_p    = dW'_p                          (only if the base is trained too),
    dA_p    = scale * B_p^T dW'_p,
    dB_p    = scale * dW'_p A_p^T,
with dW' the full weight gradient of the plain layer at W'.  The forward below does
NOT merge: it evaluates the low-rank path as its own two small products, so that the
finite-difference pins compare two independently written things.
"""
import numpy as np

from .layer import (LayerShape, RECORD_KEYS, _positions, _rms_norm, _rope, _sigmoid,
                    attention_lse, layer_backward_reuse)

PROJECTIONS = ("q", "k", "v", "o", "g", "u", "d")


def merged_weights(W, lora, scale):
    """W' = W + scale * B A for every adapted projection; gains unchanged."""
    Wm = dict(W)
    for p, (A, B) in lora.items():
        Wm["W" + p] = np.asarray(W["W" + p], dtype=np.float64) + scale * np.asarray(B, dtype=np.float64) @ np.asarray(A, dtype=np.float64)
    return Wm


def _linear(x, W, lora, scale, p):
    """x W_p^T plus the low-rank path scale * (x A_p^T) B_p^T when p carries an adapter."""
    y = x @ W["W" + p].T
    if p in lora:
        A, B = lora[p]
        y = y + scale * ((x @ np.asarray(A, dtype=np.float64).T) @ np.asarray(B, dtype=np.float64).T)
    return y


def layer_forward_lora(shape, cu_seqlens, positions, X, W, lora, scale):
    """Forward of the adapted layer.  lora: dict p -> (A_p, B_p).  Returns (Y, record)."""
    X = np.asarray(X, dtype=np.float64)
    T, H = X.shape
    Hq, Hkv, D = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    G = Hq // Hkv
    pos = _positions(cu_seqlens, positions, T)

    H1, _ = _rms_norm(X, W["g1"], shape.rms_eps)
    Q = _rope(_linear(H1, W, lora, scale, "q").reshape(T, Hq, D), pos, shape.rope_base, +1)
    K = _rope(_linear(H1, W, lora, scale, "k").reshape(T, Hkv, D), pos, shape.rope_base, +1)
    V = _linear(H1, W, lora, scale, "v").reshape(T, Hkv, D)

    LSE = attention_lse(shape, cu_seqlens, Q.reshape(T, Hq * D), K.reshape(T, Hkv * D))
    O = np.zeros((T, Hq, D), dtype=np.float64)
    for s in range(len(cu_seqlens) - 1):
        a, b = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        n = b - a
        if n == 0:
            continue
        allowed = np.tril(np.ones((n, n), dtype=bool))
        for h in range(Hq):
            sc = Q[a:b, h] @ K[a:b, h // G].T / np.sqrt(D)
            P = np.where(allowed, np.exp(sc - LSE[a:b, h][:, None]), 0.0)
            O[a:b, h] = P @ V[a:b, h // G]
    O = O.reshape(T, Hq * D)

    X2 = X + _linear(O, W, lora, scale, "o")
    H2, _ = _rms_norm(X2, W["g2"], shape.rms_eps)
    Gt = _linear(H2, W, lora, scale, "g")
    U = _linear(H2, W, lora, scale, "u")
    Act = Gt * _sigmoid(Gt) * U
    Y = X2 + _linear(Act, W, lora, scale, "d")
    rec = dict(X=X, X2=X2, Q=Q.reshape(T, Hq * D), K=K.reshape(T, Hkv * D),
               V=V.reshape(T, Hkv * D), O=O, LSE=LSE, G=Gt, U=U)
    return Y, rec


def layer_backward_reuse_lora(shape, cu_seqlens, positions, rec, W, lora, scale, dY, loss_mask=None):
    """Backward of the adapted layer from the saved record (consumed as given).

    Returns the dict of layer_backward_reuse evaluated at the merged weights (dX, dg1,
    dg2 and dW_p = dW'_p for a base that is trained too) plus dA_p, dB_p for every
    adapted projection."""
    g = layer_backward_reuse(shape, cu_seqlens, positions, rec, merged_weights(W, lora, scale), dY, loss_mask)
    for p, (A, B) in lora.items():
        dWm = g["dW" + p]
        g["dA" + p] = scale * np.asarray(B, dtype=np.float64).T @ dWm
        g["dB" + p] = scale * dWm @ np.asarray(A, dtype=np.float64).T
    return g


def stack_forward_lora(shape, cu_seqlens, positions, X0, layers_W, layers_lora, scale):
    """The adapted layers in order.  Returns (X_final, [record_l])."""
    X = np.asarray(X0, dtype=np.float64)
    recs = []
    for W, lora in zip(layers_W, layers_lora):
        X, rec = layer_forward_lora(shape, cu_seqlens, positions, X, W, lora, scale)
        recs.append(rec)
    return X, recs


def stack_backward_reuse_lora(shape, cu_seqlens, positions, recs, layers_W, layers_lora, scale, X_final,
                              g_final, W_lm, labels, loss_mask=None):
    """Cross-entropy head (Section 5) on the saved stack output, then the adapted layers from the output
    layer to the input layer (Section 4.2), each from its own saved record.  The head carries no adapter.
    Returns the dict of stack_backward_reuse; the per-layer dicts also hold dA_p, dB_p."""
    from .stack import _head_loss_and_grads
    X_final = np.asarray(X_final, dtype=np.float64)
    loss, dX, dg_final, dW_lm = _head_loss_and_grads(shape, X_final, np.asarray(g_final, dtype=np.float64),
                                                     np.asarray(W_lm, dtype=np.float64), labels, loss_mask)
    per_layer = [None] * len(layers_W)
    for l in range(len(layers_W) - 1, -1, -1):
        g = layer_backward_reuse_lora(shape, cu_seqlens, positions, recs[l], layers_W[l], layers_lora[l], scale, dX)
        dX = g["dX"]
        per_layer[l] = g
    return dict(loss=loss, dX_embed=dX, dg_final=dg_final, dW_lm=dW_lm, layers=per_layer)
