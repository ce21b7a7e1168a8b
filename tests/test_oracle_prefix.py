"""Pins for the shared-prefix layer and the DPO head of the oracle (Section 4.1, preference alignment: the
responses attend to the saved KV cache of their prompt, which chosen and rejected share; Section 6: DPO).

The shared-prefix layer is fixed by the plain layer (pinned on its own): a prompt followed by one response
is an ordinary causal sequence, and the backward pass is linear in the output gradient, so the shared batch
must equal the sum of one plain run per response.  The DPO head is fixed by finite differences, the value
log 2 at z = 0, and the pinned cross-entropy head (its gradient is a signed, scaled sum of two of those)."""
import numpy as np
import pytest

import synth_inputs as synth
from oracle import LayerShape, layer_forward, layer_backward_reuse, WEIGHT_KEYS
from oracle.prefix import (visibility, prefix_positions, layer_forward_prefix, layer_backward_reuse_prefix,
                           stack_forward_prefix, stack_backward_dpo, dpo_head)
from oracle.stack import _head_loss_and_grads


def weights(rng, shape, std=0.35):
    H, Hq, Hkv, D, F = shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn
    return dict(Wq=rng.normal(0, std, (Hq * D, H)), Wk=rng.normal(0, std, (Hkv * D, H)), Wv=rng.normal(0, std, (Hkv * D, H)),
                Wo=rng.normal(0, std, (H, Hq * D)), Wg=rng.normal(0, std, (F, H)), Wu=rng.normal(0, std, (F, H)),
                Wd=rng.normal(0, std, (H, F)), g1=1 + rng.normal(0, 0.2, H), g2=1 + rng.normal(0, 0.2, H))


SHAPE = LayerShape(16, 4, 2, 8, 24, 1e-6, 10000.0)


def test_visibility_and_positions_by_hand():
    # prompt of 3 tokens (rows 0-2), responses of 2 (rows 3-4) and 1 (row 5)
    cu, prefix = np.array([0, 3, 5, 6]), np.array([-1, 0, 0])
    want = np.array([[1, 0, 0, 0, 0, 0],
                     [1, 1, 0, 0, 0, 0],
                     [1, 1, 1, 0, 0, 0],
                     [1, 1, 1, 1, 0, 0],
                     [1, 1, 1, 1, 1, 0],
                     [1, 1, 1, 0, 0, 1]], dtype=bool)
    assert np.array_equal(visibility(cu, prefix), want)
    assert np.array_equal(prefix_positions(cu, prefix), [0, 1, 2, 3, 4, 3])


def test_no_prefix_is_the_plain_layer():
    rng = np.random.default_rng(0)
    cu = np.array([0, 4, 4, 9])
    W = weights(rng, SHAPE)
    X, R = rng.normal(size=(9, 16)), rng.normal(size=(9, 16))
    Y, rec = layer_forward_prefix(SHAPE, cu, np.array([-1, -1, -1]), X, W)
    Yp, recp = layer_forward(SHAPE, cu, None, X, W)
    np.testing.assert_allclose(Y, Yp, rtol=1e-12, atol=1e-13)
    for k in rec:
        np.testing.assert_allclose(rec[k], recp[k], rtol=1e-12, atol=1e-13, err_msg=k)
    g, gp = layer_backward_reuse_prefix(SHAPE, cu, None, rec, W, R), layer_backward_reuse(SHAPE, cu, None, recp, W, R)
    for k in gp:
        np.testing.assert_allclose(g[k], gp[k], rtol=1e-11, atol=1e-12, err_msg=k)


@pytest.mark.parametrize("P,C,Rn", [(5, 3, 4), (1, 6, 1), (7, 2, 2)])
def test_shared_prompt_equals_one_plain_sequence_per_response(P, C, Rn):
    # rows: prompt | chosen | rejected.  Plain run A = [prompt; chosen], plain run B = [prompt; rejected].
    rng = np.random.default_rng(P * 100 + C)
    W = weights(rng, SHAPE)
    cu, prefix = np.array([0, P, P + C, P + C + Rn]), np.array([-1, 0, 0])
    X = rng.normal(size=(P + C + Rn, 16))
    dY = rng.normal(size=X.shape)
    Y, rec = layer_forward_prefix(SHAPE, cu, prefix, X, W)
    XA, XB = X[:P + C], np.concatenate([X[:P], X[P + C:]])
    YA, recA = layer_forward(SHAPE, np.array([0, P + C]), None, XA, W)
    YB, recB = layer_forward(SHAPE, np.array([0, P + Rn]), None, XB, W)
    np.testing.assert_allclose(Y[:P + C], YA, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(Y[P + C:], YB[P:], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(Y[:P], YB[:P], rtol=1e-11, atol=1e-12)
    for k in rec:
        np.testing.assert_allclose(rec[k][P + C:], recB[k][P:], rtol=1e-11, atol=1e-12, err_msg=k)
    # backward: the prompt's output gradient goes to run A only; everything adds up
    g = layer_backward_reuse_prefix(SHAPE, cu, prefix, rec, W, dY)
    gA = layer_backward_reuse(SHAPE, np.array([0, P + C]), None, recA, W, dY[:P + C])
    gB = layer_backward_reuse(SHAPE, np.array([0, P + Rn]), None, recB, W,
                              np.concatenate([np.zeros((P, 16)), dY[P + C:]]))
    np.testing.assert_allclose(g["dX"][:P], gA["dX"][:P] + gB["dX"][:P], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["dX"][P:P + C], gA["dX"][P:], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["dX"][P + C:], gB["dX"][P:], rtol=1e-10, atol=1e-12)
    for k in WEIGHT_KEYS:
        np.testing.assert_allclose(g["d" + k], gA["d" + k] + gB["d" + k], rtol=1e-10, atol=1e-11, err_msg=k)


def test_layer_gradients_by_finite_differences_two_groups():
    rng = np.random.default_rng(3)
    b = synth.preference_batch([4, 2], [[3, 2], [1, 4]], 11, 0)
    cu, prefix = b["cu"], b["prefix"]
    assert np.array_equal(prefix_positions(cu, prefix), b["positions"])
    T = int(cu[-1])
    W = weights(rng, SHAPE)
    X, R = rng.normal(size=(T, 16)), rng.normal(size=(T, 16))
    _, rec = layer_forward_prefix(SHAPE, cu, prefix, X, W)
    g = layer_backward_reuse_prefix(SHAPE, cu, prefix, rec, W, R)

    def loss():
        return float(np.sum(layer_forward_prefix(SHAPE, cu, prefix, X, W)[0] * R))
    h = 1e-5
    for name, Pm in [("dX", X)] + [("d" + k, W[k]) for k in WEIGHT_KEYS]:
        an = g[name]
        idx = list(np.ndindex(*Pm.shape))
        idx = [idx[i] for i in rng.choice(len(idx), min(40, len(idx)), replace=False)]
        ref = max(np.abs(an).max(), 1e-30)
        for i in idx:
            old = Pm[i]
            Pm[i] = old + h
            fp = loss()
            Pm[i] = old - h
            fm = loss()
            Pm[i] = old
            assert abs((fp - fm) / (2 * h) - an[i]) <= 2e-6 * ref, (name, i)


def head_case(seed, V=13):
    rng = np.random.default_rng(seed)
    b = synth.preference_batch([4, 3], [[3, 2], [2, 5]], V, seed)
    T = int(b["cu"][-1])
    Xf = rng.normal(size=(T, 16))
    gf = 1 + 0.1 * rng.normal(size=16)
    Wlm = rng.normal(0, 0.4, (V, 16))
    ref = rng.normal(0, 1.0, 4)
    return b, Xf, gf, Wlm, ref


def test_items_of_the_generator():
    b = synth.preference_batch([4, 3], [[3, 2], [2, 5]], 13, 1)
    cu, tok = b["cu"], b["tokens"]
    assert list(b["prefix"]) == [-1, -1, 0, 0, 1, 1]
    # one item per response token; the first one sits on the last prompt row
    assert len(b["item_row"]) == 3 + 2 + 2 + 5
    assert np.all(np.diff(b["item_row"]) >= 0)
    for s, g in ((2, 0), (3, 0), (4, 1), (5, 1)):
        sel = b["item_slot"] == s - 2
        rows, labels = b["item_row"][sel], b["item_label"][sel]
        n = cu[s + 1] - cu[s]
        assert list(rows) == [cu[g + 1] - 1] + list(range(cu[s], cu[s] + n - 1))
        assert list(labels) == list(tok[cu[s]:cu[s + 1]])


def test_dpo_value_at_zero_margin_and_antisymmetry():
    b, Xf, gf, Wlm, _ = head_case(2)
    # reference equal to the policy: z = 0, loss = log 2
    loss0, _, _, _, z0 = dpo_head(SHAPE, Xf, gf, Wlm, b["item_row"], b["item_label"], b["item_slot"], np.zeros(4), 0.3)
    margin = z0 / 0.3   # with ref = 0: z = beta (pi_c - pi_r); a reference with the same margin gives z = 0
    ref = np.zeros(4)
    ref[0::2] = margin
    loss, _, _, _, z = dpo_head(SHAPE, Xf, gf, Wlm, b["item_row"], b["item_label"], b["item_slot"], ref, 0.3)
    np.testing.assert_allclose(z, 0.0, atol=1e-12)
    assert abs(loss - np.log(2.0)) < 1e-12
    # exchanging chosen and rejected negates z, and -log sigmoid(z) - (-log sigmoid(-z)) = -z
    swapped = b["item_slot"] ^ 1
    loss_s, _, _, _, z_s = dpo_head(SHAPE, Xf, gf, Wlm, b["item_row"], b["item_label"], swapped, np.zeros(4), 0.3)
    np.testing.assert_allclose(z_s, -z0, rtol=1e-12)
    assert abs((loss0 - loss_s) - np.mean(-z0)) < 1e-12


def test_dpo_gradient_is_a_signed_sum_of_cross_entropy_gradients():
    # one pair whose items sit on distinct rows: d loss = beta sigmoid(-z) (d CEsum_chosen - d CEsum_rejected)
    rng = np.random.default_rng(5)
    T, V, beta = 9, 7, 0.7
    Xf, gf, Wlm = rng.normal(size=(T, 16)), 1 + 0.1 * rng.normal(size=16), rng.normal(0, 0.4, (V, 16))
    rows = np.array([1, 2, 3, 5, 6, 8])
    labels = rng.integers(0, V, 6)
    slots = np.array([0, 0, 0, 1, 1, 1])
    ref = np.array([0.4, -0.2])
    loss, dX, dg, dW, z = dpo_head(SHAPE, Xf, gf, Wlm, rows, labels, slots, ref, beta)
    parts = []
    for s in (0, 1):
        lab = np.full(T, -1)
        lab[rows[slots == s]] = labels[slots == s]
        ce, dXc, dgc, dWc = _head_loss_and_grads(SHAPE, Xf, gf, Wlm, lab, None)
        parts.append((3 * ce, 3 * dXc, 3 * dgc, 3 * dWc))    # mean over 3 counted rows -> sum
    z_want = beta * ((-parts[0][0] - ref[0]) - (-parts[1][0] - ref[1]))
    assert abs(z[0] - z_want) < 1e-12
    assert abs(loss - np.log1p(np.exp(-z_want))) < 1e-12
    c = beta / (1.0 + np.exp(z_want))
    np.testing.assert_allclose(dX, c * (parts[0][1] - parts[1][1]), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dg, c * (parts[0][2] - parts[1][2]), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dW, c * (parts[0][3] - parts[1][3]), rtol=1e-10, atol=1e-13)


def test_dpo_head_finite_differences_with_a_shared_row():
    b, Xf, gf, Wlm, ref = head_case(4)
    args = (b["item_row"], b["item_label"], b["item_slot"], ref, 0.5)
    loss, dX, dg, dW, _ = dpo_head(SHAPE, Xf, gf, Wlm, *args)
    assert np.sum(b["item_row"] == b["cu"][1] - 1) == 2       # last row of prompt 0 scores two tokens
    rng = np.random.default_rng(1)
    h = 1e-6
    for an, Pm in ((dX, Xf), (dg, gf), (dW, Wlm)):
        idx = list(np.ndindex(*Pm.shape))
        ref_mag = max(np.abs(an).max(), 1e-30)
        for i in [idx[k] for k in rng.choice(len(idx), min(50, len(idx)), replace=False)]:
            old = Pm[i]
            Pm[i] = old + h
            fp = dpo_head(SHAPE, Xf, gf, Wlm, *args)[0]
            Pm[i] = old - h
            fm = dpo_head(SHAPE, Xf, gf, Wlm, *args)[0]
            Pm[i] = old
            assert abs((fp - fm) / (2 * h) - an[i]) <= 1e-5 * ref_mag, i
    # rows that score nothing receive no gradient
    unscored = np.setdiff1d(np.arange(Xf.shape[0]), b["item_row"])
    assert np.all(dX[unscored] == 0)


def test_stack_dpo_finite_differences_through_the_shared_prompt():
    # two layers; weights of layer 0 reach the loss through the prompt's keys and values as well
    rng = np.random.default_rng(8)
    b, _, gf, Wlm, ref = head_case(6)
    cu, prefix = b["cu"], b["prefix"]
    T = int(cu[-1])
    Ws = [weights(rng, SHAPE), weights(rng, SHAPE)]
    X0 = rng.normal(size=(T, 16))
    items = (b["item_row"], b["item_label"], b["item_slot"])

    def loss():
        Xf, _ = stack_forward_prefix(SHAPE, cu, prefix, X0, Ws)
        return dpo_head(SHAPE, Xf, gf, Wlm, *items, ref, 0.5)[0]

    Xf, recs = stack_forward_prefix(SHAPE, cu, prefix, X0, Ws)
    g = stack_backward_dpo(SHAPE, cu, prefix, recs, Ws, Xf, gf, Wlm, *items, ref, 0.5)
    assert abs(g["loss"] - loss()) < 1e-12
    assert np.abs(g["dX_embed"][:b["cu"][2]]).min() > 0      # prompt rows do receive gradient
    h = 1e-5
    checks = [(g["dX_embed"], X0)] + [(g["layers"][l]["d" + k], Ws[l][k]) for l in (0, 1) for k in ("Wk", "Wv", "Wq", "Wd", "g1")]
    for an, Pm in checks:
        idx = list(np.ndindex(*Pm.shape))
        ref_mag = max(np.abs(an).max(), 1e-30)
        for i in [idx[k] for k in rng.choice(len(idx), min(15, len(idx)), replace=False)]:
            old = Pm[i]
            Pm[i] = old + h
            fp = loss()
            Pm[i] = old - h
            fm = loss()
            Pm[i] = old
            assert abs((fp - fm) / (2 * h) - an[i]) <= 1e-5 * ref_mag, i


def test_stack_dpo_adapter_gradients_by_finite_differences():
    # adapters on both layers; the loss is evaluated by the shared-prefix forward at the merged weights
    from oracle.lora import merged_weights
    from oracle.prefix import stack_backward_dpo_lora
    rng = np.random.default_rng(18)
    b, _, gf, Wlm, ref = head_case(7)
    cu, prefix = b["cu"], b["prefix"]
    T = int(cu[-1])
    Ws = [weights(rng, SHAPE), weights(rng, SHAPE)]
    r = 2
    loras = [{p: (rng.normal(0, 0.4, (r, W["W" + p].shape[1])), rng.normal(0, 0.4, (W["W" + p].shape[0], r)))
              for p in proj} for W, proj in zip(Ws, (("q", "k", "d"), ("v", "o", "g", "u")))]
    X0 = rng.normal(size=(T, 16))
    items = (b["item_row"], b["item_label"], b["item_slot"])
    scale = 0.6

    def forward():
        return stack_forward_prefix(SHAPE, cu, prefix, X0, [merged_weights(W, lo, scale) for W, lo in zip(Ws, loras)])

    def loss():
        return dpo_head(SHAPE, forward()[0], gf, Wlm, *items, ref, 0.5)[0]

    Xf, recs = forward()
    g = stack_backward_dpo_lora(SHAPE, cu, prefix, recs, Ws, loras, scale, Xf, gf, Wlm, *items, ref, 0.5)
    h = 1e-5
    for l, lo in enumerate(loras):
        for p, (A, B) in lo.items():
            for name, Pm in (("dA" + p, A), ("dB" + p, B)):
                an = g["layers"][l][name]
                ref_mag = max(np.abs(an).max(), 1e-30)
                idx = list(np.ndindex(*Pm.shape))
                for i in [idx[k] for k in rng.choice(len(idx), min(8, len(idx)), replace=False)]:
                    old = Pm[i]
                    Pm[i] = old + h
                    fp = loss()
                    Pm[i] = old - h
                    fm = loss()
                    Pm[i] = old
                    assert abs((fp - fm) / (2 * h) - an[i]) <= 1e-5 * ref_mag, (l, name, i)
