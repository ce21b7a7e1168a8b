"""Pins for the low-rank-adapter oracle (Section 3 assumption A1, Section 6 "Training": rank-8 LoRA).

The backward is defined through the merged weights; the forward evaluates the low-rank path
separately.  Finite differences of that forward, the special cases B = 0, scale = 0 and A = identity
(where the adapter is an ordinary dense weight), and the plain-layer oracle (pinned elsewhere) fix it."""
import numpy as np
import pytest

from oracle import LayerShape, layer_forward, layer_backward_reuse
from oracle.lora import PROJECTIONS, layer_forward_lora, layer_backward_reuse_lora, merged_weights


def make(seed, H=16, Hq=4, Hkv=2, D=8, F=24, lens=(1, 5, 8), r=3, adapted=PROJECTIONS, wstd=0.35):
    rng = np.random.default_rng(seed)
    shape = LayerShape(H, Hq, Hkv, D, F, 1e-6, 10000.0)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    T = int(cu[-1])
    W = dict(Wq=rng.normal(0, wstd, (Hq * D, H)), Wk=rng.normal(0, wstd, (Hkv * D, H)),
             Wv=rng.normal(0, wstd, (Hkv * D, H)), Wo=rng.normal(0, wstd, (H, Hq * D)),
             Wg=rng.normal(0, wstd, (F, H)), Wu=rng.normal(0, wstd, (F, H)),
             Wd=rng.normal(0, wstd, (H, F)), g1=1 + rng.normal(0, 0.2, H), g2=1 + rng.normal(0, 0.2, H))
    lora = {p: (rng.normal(0, 0.4, (r, W["W" + p].shape[1])), rng.normal(0, 0.4, (W["W" + p].shape[0], r)))
            for p in adapted}
    X = rng.normal(0, 1, (T, H))
    R = rng.normal(0, 1, (T, H))
    return shape, cu, T, W, lora, X, R


@pytest.mark.parametrize("seed,cfg", [(0, dict()), (1, dict(Hq=2, Hkv=2, lens=(7,), r=2, adapted=("q", "v"))),
                                      (2, dict(Hq=6, Hkv=2, D=4, F=20, lens=(3, 1, 6), r=4, adapted=("k", "o", "g", "d")))])
def test_finite_differences_of_the_unmerged_forward(seed, cfg):
    shape, cu, T, W, lora, X, R = make(seed, **cfg)
    scale = 0.7
    _, rec = layer_forward_lora(shape, cu, None, X, W, lora, scale)
    g = layer_backward_reuse_lora(shape, cu, None, rec, W, lora, scale, R)

    def loss():
        Y, _ = layer_forward_lora(shape, cu, None, X, W, lora, scale)
        return float(np.sum(Y * R))

    rng = np.random.default_rng(50 + seed)
    h = 1e-5
    tensors = {"dX": X}
    for p, (A, B) in lora.items():
        tensors["dA" + p] = A
        tensors["dB" + p] = B
    for p in PROJECTIONS:  # the base weight gradient is the merged-weight gradient
        tensors["dW" + p] = W["W" + p]
    for name, P in tensors.items():
        an = g[name]
        assert an.shape == P.shape, name
        idx = list(np.ndindex(*P.shape))
        if len(idx) > 60:
            idx = [idx[i] for i in rng.choice(len(idx), 60, replace=False)]
        ref = max(np.abs(an).max(), 1e-30)
        for i in idx:
            old = P[i]
            P[i] = old + h
            fp = loss()
            P[i] = old - h
            fm = loss()
            P[i] = old
            assert abs((fp - fm) / (2 * h) - an[i]) <= 2e-6 * ref, (name, i)


def test_projection_without_adapter_has_no_adapter_gradient():
    shape, cu, T, W, lora, X, R = make(3, adapted=("q", "v"))
    _, rec = layer_forward_lora(shape, cu, None, X, W, lora, 1.0)
    g = layer_backward_reuse_lora(shape, cu, None, rec, W, lora, 1.0, R)
    assert sorted(k for k in g if k.startswith(("dA", "dB"))) == ["dAq", "dAv", "dBq", "dBv"]


def test_zero_scale_and_zero_B_reduce_to_the_plain_layer():
    shape, cu, T, W, lora, X, R = make(4)
    Yp, recp = layer_forward(shape, cu, None, X, W)
    gp = layer_backward_reuse(shape, cu, None, recp, W, R)
    # scale = 0: the adapter is absent from the function
    Y0, rec0 = layer_forward_lora(shape, cu, None, X, W, lora, 0.0)
    np.testing.assert_allclose(Y0, Yp, rtol=0, atol=1e-12)
    g0 = layer_backward_reuse_lora(shape, cu, None, rec0, W, lora, 0.0, R)
    np.testing.assert_allclose(g0["dX"], gp["dX"], rtol=0, atol=1e-12)
    for p in PROJECTIONS:
        assert np.all(g0["dA" + p] == 0) and np.all(g0["dB" + p] == 0)
    # B = 0 (the usual initialisation): same function, dA = 0, dB = scale * dW A^T with the plain dW
    lora0 = {p: (A, np.zeros_like(B)) for p, (A, B) in lora.items()}
    Yb, recb = layer_forward_lora(shape, cu, None, X, W, lora0, 0.5)
    np.testing.assert_allclose(Yb, Yp, rtol=0, atol=1e-12)
    gb = layer_backward_reuse_lora(shape, cu, None, recb, W, lora0, 0.5, R)
    for p in PROJECTIONS:
        assert np.all(gb["dA" + p] == 0)
        np.testing.assert_allclose(gb["dB" + p], 0.5 * gp["dW" + p] @ lora[p][0].T, rtol=1e-10, atol=1e-12)


def test_identity_A_makes_the_adapter_a_dense_weight():
    # r = in, A = I: y = x (W + scale B)^T, so dB = scale * dW of the plain layer at weight W + scale B
    shape, cu, T, W, _, X, R = make(5)
    rng = np.random.default_rng(9)
    scale = 0.3
    B = rng.normal(0, 0.3, W["Wg"].shape)
    lora = {"g": (np.eye(shape.hidden), B)}
    Y, rec = layer_forward_lora(shape, cu, None, X, W, lora, scale)
    W2 = dict(W, Wg=W["Wg"] + scale * B)
    Y2, rec2 = layer_forward(shape, cu, None, X, W2)
    np.testing.assert_allclose(Y, Y2, rtol=1e-11, atol=1e-12)
    g = layer_backward_reuse_lora(shape, cu, None, rec, W, lora, scale, R)
    g2 = layer_backward_reuse(shape, cu, None, rec2, W2, R)
    np.testing.assert_allclose(g["dBg"], scale * g2["dWg"], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["dX"], g2["dX"], rtol=1e-10, atol=1e-12)


def test_merged_weights_reproduce_the_adapted_forward():
    shape, cu, T, W, lora, X, R = make(6)
    Y, _ = layer_forward_lora(shape, cu, None, X, W, lora, 1.3)
    Ym, _ = layer_forward(shape, cu, None, X, merged_weights(W, lora, 1.3))
    np.testing.assert_allclose(Y, Ym, rtol=1e-10, atol=1e-11)


def test_loss_mask_equals_zeroed_rows():
    shape, cu, T, W, lora, X, R = make(7)
    _, rec = layer_forward_lora(shape, cu, None, X, W, lora, 1.0)
    mask = (np.random.default_rng(3).random(T) < 0.5).astype(np.uint8)
    a = layer_backward_reuse_lora(shape, cu, None, rec, W, lora, 1.0, R, loss_mask=mask)
    Rz = R.copy()
    Rz[mask == 0] = 0
    b = layer_backward_reuse_lora(shape, cu, None, rec, W, lora, 1.0, Rz)
    for k in a:
        assert np.array_equal(a[k], b[k]), k


def test_stack_adapter_gradients_by_finite_differences_of_the_loss():
    # two adapted layers + head: d loss / d A, d B of BOTH layers against central differences of the
    # scalar loss computed by the unmerged forward (the gradient of layer 0 passes through layer 1)
    from oracle.lora import stack_forward_lora, stack_backward_reuse_lora
    from oracle.stack import _head_loss_and_grads
    shape, cu, T, W0, l0, X, _ = make(11, adapted=("q", "o", "d"), r=2)
    _, _, _, W1, l1, _, _ = make(12, adapted=("k", "g"), r=2)
    rng = np.random.default_rng(5)
    V = 13
    gf = 1 + 0.1 * rng.normal(size=shape.hidden)
    Wlm = rng.normal(0, 0.3, (V, shape.hidden))
    labels = rng.integers(0, V, T)
    labels[cu[1:] - 1] = -1
    scale = 0.8
    Ws, Ls = [W0, W1], [l0, l1]

    def loss():
        Xf, _ = stack_forward_lora(shape, cu, None, X, Ws, Ls, scale)
        return _head_loss_and_grads(shape, Xf, gf, Wlm, labels, None)[0]

    Xf, recs = stack_forward_lora(shape, cu, None, X, Ws, Ls, scale)
    g = stack_backward_reuse_lora(shape, cu, None, recs, Ws, Ls, scale, Xf, gf, Wlm, labels)
    assert abs(g["loss"] - loss()) < 1e-12
    h = 1e-5
    for l, lora in enumerate(Ls):
        for p, (A, B) in lora.items():
            for name, P in (("dA" + p, A), ("dB" + p, B)):
                an = g["layers"][l][name]
                ref = max(np.abs(an).max(), 1e-30)
                idx = list(np.ndindex(*P.shape))
                for i in [idx[k] for k in rng.choice(len(idx), min(12, len(idx)), replace=False)]:
                    old = P[i]
                    P[i] = old + h
                    fp = loss()
                    P[i] = old - h
                    fm = loss()
                    P[i] = old
                    assert abs((fp - fm) / (2 * h) - an[i]) <= 5e-6 * ref, (l, name, i)
