"""Oracle for the L-layer stack with final RMSNorm, LM head and cross-entropy.

Test infrastructure only (see the package docstring).  float64 throughout.

Paper basis: Section 5 (the continual-pre-training loss is cross-entropy over the
prefill output and the prompt text), Section 4.2 / 4.3.2 (backward walks the layers
from the output layer to the input layer, each consuming its own saved
activations).  Readings where the paper is silent: the loss is the mean negative
log-likelihood over counted positions; a position counts when its label is >= 0
and its loss-mask byte (if a mask is given) is nonzero; with no counted position
the loss and every gradient are zero.
"""
import numpy as np
from .layer import (layer_forward, layer_backward_reuse, _rms_norm, _rms_norm_backward)


def stack_forward(shape, cu_seqlens, positions, X0, layers_W):
    """Runs the layers in order.  Returns (X_final, [record_l])."""
    X = np.asarray(X0, dtype=np.float64)
    recs = []
    for W in layers_W:
        X, rec = layer_forward(shape, cu_seqlens, positions, X, W)
        recs.append(rec)
    return X, recs


def _head_loss_and_grads(shape, X_final, g_final, W_lm, labels, loss_mask):
    T, H = X_final.shape
    labels = np.asarray(labels, dtype=np.int64)
    counted = labels >= 0
    if loss_mask is not None:
        counted &= (np.asarray(loss_mask) != 0)
    N = int(np.sum(counted))
    Hf, rf = _rms_norm(X_final, g_final, shape.rms_eps)
    dX_final = np.zeros_like(X_final)
    dg_final = np.zeros_like(g_final)
    dW_lm = np.zeros_like(W_lm)
    if N == 0:
        return 0.0, dX_final, dg_final, dW_lm
    logits = Hf @ W_lm.T
    m = logits.max(axis=1, keepdims=True)
    logZ = m + np.log(np.sum(np.exp(logits - m), axis=1, keepdims=True))
    logp = logits - logZ
    rows = np.flatnonzero(counted)
    loss = -np.sum(logp[rows, labels[rows]]) / N
    dlogits = np.zeros_like(logits)
    dlogits[rows] = np.exp(logp[rows])
    dlogits[rows, labels[rows]] -= 1.0
    dlogits /= N
    dW_lm = dlogits.T @ Hf
    dHf = dlogits @ W_lm
    dX_final, dg_final = _rms_norm_backward(dHf, X_final, g_final, rf)
    return float(loss), dX_final, dg_final, dW_lm


def stack_backward_reuse(shape, cu_seqlens, positions, recs, layers_W, X_final, g_final, W_lm,
                         labels, loss_mask=None):
    """Loss and gradients from saved per-layer records plus the saved stack output.

    Returns dict: loss, dX_embed [T,H] (gradient w.r.t. the input of layer 0),
    dg_final, dW_lm, layers = [per-layer gradient dicts as layer_backward_reuse].
    """
    X_final = np.asarray(X_final, dtype=np.float64)
    loss, dX, dg_final, dW_lm = _head_loss_and_grads(shape, X_final, g_final, W_lm, labels, loss_mask)
    per_layer = [None] * len(layers_W)
    for l in range(len(layers_W) - 1, -1, -1):
        g = layer_backward_reuse(shape, cu_seqlens, positions, recs[l], layers_W[l], dX)
        dX = g["dX"]
        per_layer[l] = g
    return dict(loss=loss, dX_embed=dX, dg_final=dg_final, dW_lm=dW_lm, layers=per_layer)


def stack_backward_recompute(shape, cu_seqlens, positions, X0, layers_W, g_final, W_lm, labels,
                             loss_mask=None):
    """Comparison path: recompute the whole forward from X0, then back-propagate."""
    X_final, recs = stack_forward(shape, cu_seqlens, positions, X0, layers_W)
    return stack_backward_reuse(shape, cu_seqlens, positions, recs, layers_W, X_final, g_final,
                                W_lm, labels, loss_mask)


def stack_loss(shape, cu_seqlens, positions, X0, layers_W, g_final, W_lm, labels, loss_mask=None):
    """Scalar loss only (used by finite-difference pins)."""
    X_final, _ = stack_forward(shape, cu_seqlens, positions, X0, layers_W)
    loss, _, _, _ = _head_loss_and_grads(shape, X_final, np.asarray(g_final, dtype=np.float64),
                                         np.asarray(W_lm, dtype=np.float64), labels, loss_mask)
    return loss
