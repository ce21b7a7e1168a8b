"""Pins for the stack oracle (Section 5: cross-entropy on the prefill output;
Section 4.3.2: layers are walked output -> input)."""
import numpy as np
import pytest

from oracle import LayerShape, stack_forward, stack_backward_reuse, stack_backward_recompute
from oracle.stack import stack_loss


def make(seed, L=2, V=11, H=8, Hq=2, Hkv=1, D=4, F=12, lens=(4, 1, 6)):
    rng = np.random.default_rng(seed)
    shape = LayerShape(H, Hq, Hkv, D, F, 1e-6, 10000.0)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    T = int(cu[-1])
    std = 0.4
    Ws = [dict(Wq=rng.normal(0, std, (Hq * D, H)), Wk=rng.normal(0, std, (Hkv * D, H)),
               Wv=rng.normal(0, std, (Hkv * D, H)), Wo=rng.normal(0, std, (H, Hq * D)),
               Wg=rng.normal(0, std, (F, H)), Wu=rng.normal(0, std, (F, H)), Wd=rng.normal(0, std, (H, F)),
               g1=1 + rng.normal(0, 0.1, H), g2=1 + rng.normal(0, 0.1, H)) for _ in range(L)]
    X0 = rng.normal(0, 1, (T, H))
    gf = 1 + rng.normal(0, 0.1, H)
    Wlm = rng.normal(0, std, (V, H))
    ids = rng.integers(0, V, T)
    labels = np.full(T, -1, dtype=np.int64)
    for s in range(len(lens)):
        a, b = cu[s], cu[s + 1]
        labels[a:b - 1] = ids[a + 1:b]          # next-token labels, last position ignored
    return shape, cu, T, Ws, X0, gf, Wlm, labels


def test_stack_finite_differences():
    shape, cu, T, Ws, X0, gf, Wlm, labels = make(0)
    mask = np.ones(T, np.uint8); mask[2] = 0
    g = stack_backward_recompute(shape, cu, None, X0, Ws, gf, Wlm, labels, mask)
    rng = np.random.default_rng(1)
    h = 1e-5
    f = lambda: stack_loss(shape, cu, None, X0, Ws, gf, Wlm, labels, mask)
    assert abs(f() - g["loss"]) < 1e-13
    targets = [("dX_embed", X0, g["dX_embed"]), ("dg_final", gf, g["dg_final"]), ("dW_lm", Wlm, g["dW_lm"])]
    for l in range(len(Ws)):
        for k in Ws[l]:
            targets.append((f"L{l}.d{k}", Ws[l][k], g["layers"][l]["d" + k]))
    for name, P, an in targets:
        scale = max(np.abs(an).max(), 1e-30)
        idx = list(np.ndindex(*P.shape))
        for i in [idx[j] for j in rng.choice(len(idx), min(12, len(idx)), replace=False)]:
            old = P[i]
            P[i] = old + h; fp = f()
            P[i] = old - h; fm = f()
            P[i] = old
            assert abs((fp - fm) / (2 * h) - an[i]) <= 1e-6 * scale, (name, i)
        d = rng.normal(0, 1, P.shape)
        P += h * d; fp = f()
        P -= 2 * h * d; fm = f()
        P += h * d
        assert abs((fp - fm) / (2 * h) - np.sum(an * d)) <= 1e-6 * max(abs(np.sum(an * d)), scale), name


def test_stack_reuse_equals_recompute_and_layer_order():
    shape, cu, T, Ws, X0, gf, Wlm, labels = make(2, L=3)
    Xf, recs = stack_forward(shape, cu, None, X0, Ws)
    a = stack_backward_reuse(shape, cu, None, recs, Ws, Xf, gf, Wlm, labels)
    b = stack_backward_recompute(shape, cu, None, X0, Ws, gf, Wlm, labels)
    assert abs(a["loss"] - b["loss"]) < 1e-13
    assert np.allclose(a["dX_embed"], b["dX_embed"], rtol=1e-12, atol=1e-15)
    # records are per layer: swapping two layers' records must change the result
    sw = [recs[1], recs[0], recs[2]]
    c = stack_backward_reuse(shape, cu, None, sw, Ws, Xf, gf, Wlm, labels)
    assert np.max(np.abs(c["dX_embed"] - a["dX_embed"])) > 1e-8


def test_loss_closed_forms():
    shape, cu, T, Ws, X0, gf, Wlm, labels = make(3)
    V = Wlm.shape[0]
    # zero LM head => uniform distribution => loss = ln V exactly
    g = stack_backward_recompute(shape, cu, None, X0, Ws, gf, np.zeros_like(Wlm), labels)
    assert abs(g["loss"] - np.log(V)) < 1e-13
    assert np.max(np.abs(g["dX_embed"])) == 0
    # every row of dlogits sums to zero => each column sum of dW_lm^T ... : sum_v dW_lm[v,:] = 0
    g = stack_backward_recompute(shape, cu, None, X0, Ws, gf, Wlm, labels)
    assert np.max(np.abs(g["dW_lm"].sum(axis=0))) < 1e-13
    # nothing counted => zero loss and zero gradients
    z = stack_backward_recompute(shape, cu, None, X0, Ws, gf, Wlm, np.full(T, -1))
    assert z["loss"] == 0.0 and np.max(np.abs(z["dX_embed"])) == 0 and np.max(np.abs(z["dW_lm"])) == 0
    z = stack_backward_recompute(shape, cu, None, X0, Ws, gf, Wlm, labels, np.zeros(T, np.uint8))
    assert z["loss"] == 0.0 and np.max(np.abs(z["layers"][0]["dWq"])) == 0
    # one counted position: loss = -log softmax(logits)[label] of that row alone (mean over 1)
    one = np.full(T, -1); one[5] = labels[5]
    g1 = stack_backward_recompute(shape, cu, None, X0, Ws, gf, Wlm, one)
    # and the mean over two disjoint singletons is their average
    two = np.full(T, -1); two[7] = labels[7]
    g2 = stack_backward_recompute(shape, cu, None, X0, Ws, gf, Wlm, two)
    both = np.full(T, -1); both[5] = labels[5]; both[7] = labels[7]
    g12 = stack_backward_recompute(shape, cu, None, X0, Ws, gf, Wlm, both)
    assert abs(g12["loss"] - 0.5 * (g1["loss"] + g2["loss"])) < 1e-13
    assert np.allclose(g12["dW_lm"], 0.5 * (g1["dW_lm"] + g2["dW_lm"]), rtol=1e-12, atol=1e-15)
