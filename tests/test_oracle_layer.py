"""Pins for the decoder-layer oracle (none of them re-types its formulas):
finite differences, the reuse == recompute invariant of Section 1 / Section 2.5.1,
a library attention routine under autograd, closed forms and special cases."""
import numpy as np
import pytest
import torch

from oracle import (LayerShape, layer_forward, layer_backward_reuse, layer_backward_recompute,
                    attention_lse, RECORD_KEYS, WEIGHT_KEYS)
from oracle.layer import attention_backward, layer_backward_reuse_tail_rows, _rope, _rms_norm, _rms_norm_backward

GRADS = ("dX",) + tuple("d" + k for k in WEIGHT_KEYS)


def make(seed, H=16, Hq=4, Hkv=2, D=8, F=24, lens=(1, 5, 8), wstd=0.35, eps=1e-6):
    rng = np.random.default_rng(seed)
    shape = LayerShape(H, Hq, Hkv, D, F, eps, 10000.0)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    T = int(cu[-1])
    W = dict(Wq=rng.normal(0, wstd, (Hq * D, H)), Wk=rng.normal(0, wstd, (Hkv * D, H)),
             Wv=rng.normal(0, wstd, (Hkv * D, H)), Wo=rng.normal(0, wstd, (H, Hq * D)),
             Wg=rng.normal(0, wstd, (F, H)), Wu=rng.normal(0, wstd, (F, H)),
             Wd=rng.normal(0, wstd, (H, F)), g1=1 + rng.normal(0, 0.2, H), g2=1 + rng.normal(0, 0.2, H))
    X = rng.normal(0, 1, (T, H))
    R = rng.normal(0, 1, (T, H))
    return shape, cu, T, W, X, R


def scalar(shape, cu, X, W, R, positions=None):
    Y, _ = layer_forward(shape, cu, positions, X, W)
    return float(np.sum(Y * R))


@pytest.mark.parametrize("seed,cfg", [(0, dict()), (1, dict(Hq=2, Hkv=2, D=8, lens=(8,))),
                                      (2, dict(Hq=6, Hkv=2, D=4, F=20, lens=(3, 1, 1, 6)))])
def test_finite_differences_all_gradients(seed, cfg):
    shape, cu, T, W, X, R = make(seed, **cfg)
    Y, rec = layer_forward(shape, cu, None, X, W)
    g = layer_backward_reuse(shape, cu, None, rec, W, R)
    rng = np.random.default_rng(100 + seed)
    h = 1e-5
    params = dict(W, X=X)
    for name, P in params.items():
        an = g["d" + name]
        assert an.shape == P.shape
        idx = list(np.ndindex(*P.shape))
        if len(idx) > 160:
            idx = [idx[i] for i in rng.choice(len(idx), 160, replace=False)]
        scale = max(np.abs(an).max(), 1e-30)
        for i in idx:
            old = P[i]
            P[i] = old + h
            fp = scalar(shape, cu, params["X"], W, R)
            P[i] = old - h
            fm = scalar(shape, cu, params["X"], W, R)
            P[i] = old
            fd = (fp - fm) / (2 * h)
            assert abs(fd - an[i]) <= 1e-6 * scale, (name, i, fd, an[i])
        # one random direction per tensor covers every coordinate in aggregate
        d = rng.normal(0, 1, P.shape)
        P += h * d
        fp = scalar(shape, cu, params["X"], W, R)
        P -= 2 * h * d
        fm = scalar(shape, cu, params["X"], W, R)
        P += h * d
        assert abs((fp - fm) / (2 * h) - np.sum(an * d)) <= 1e-6 * max(abs(np.sum(an * d)), scale)


def test_finite_differences_custom_positions():
    shape, cu, T, W, X, R = make(7)
    pos = np.random.default_rng(7).integers(0, 50, T)
    Y, rec = layer_forward(shape, cu, pos, X, W)
    g = layer_backward_reuse(shape, cu, pos, rec, W, R)
    rng = np.random.default_rng(8)
    h = 1e-5
    for name, P in dict(Wq=W["Wq"], Wk=W["Wk"], X=X).items():
        d = rng.normal(0, 1, P.shape)
        P += h * d
        fp = scalar(shape, cu, X, W, R, pos)
        P -= 2 * h * d
        fm = scalar(shape, cu, X, W, R, pos)
        P += h * d
        an = np.sum(g["d" + name] * d)
        assert abs((fp - fm) / (2 * h) - an) <= 1e-6 * max(abs(an), 1e-3)


def test_reuse_equals_recompute_and_every_saved_tensor_is_consumed():
    shape, cu, T, W, X, R = make(3)
    _, rec = layer_forward(shape, cu, None, X, W)
    a = layer_backward_reuse(shape, cu, None, rec, W, R)
    b = layer_backward_recompute(shape, cu, None, X, W, R)
    for k in GRADS:
        assert np.max(np.abs(a[k] - b[k])) <= 1e-12 * max(1.0, np.abs(b[k]).max()), k
    # perturbing any one saved tensor must change the result: the reuse path may not
    # silently recompute it from X and the weights
    rng = np.random.default_rng(4)
    for key in RECORD_KEYS:
        bad = dict(rec)
        bad[key] = rec[key] + 0.05 * rng.normal(0, 1, rec[key].shape)
        c = layer_backward_reuse(shape, cu, None, bad, W, R)
        assert max(np.max(np.abs(c[k] - a[k])) for k in GRADS) > 1e-6, key


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (4, 2), (6, 1)])
def test_attention_backward_against_library_sdpa_autograd(Hq, Hkv):
    D, n = 8, 7
    shape = LayerShape(16, Hq, Hkv, D, 8)
    rng = np.random.default_rng(Hq * 10 + Hkv)
    cu = np.array([0, n, n + 3])
    T = n + 3
    Q, K, V = rng.normal(0, 1, (T, Hq * D)), rng.normal(0, 1, (T, Hkv * D)), rng.normal(0, 1, (T, Hkv * D))
    dO = rng.normal(0, 1, (T, Hq * D))
    tq = torch.tensor(Q, dtype=torch.float64, requires_grad=True)
    tk = torch.tensor(K, dtype=torch.float64, requires_grad=True)
    tv = torch.tensor(V, dtype=torch.float64, requires_grad=True)
    outs = []
    for s in range(2):
        a, b = int(cu[s]), int(cu[s + 1])
        q = tq[a:b].reshape(b - a, Hq, D).transpose(0, 1)[None]
        k = tk[a:b].reshape(b - a, Hkv, D).transpose(0, 1).repeat_interleave(Hq // Hkv, dim=0)[None]
        v = tv[a:b].reshape(b - a, Hkv, D).transpose(0, 1).repeat_interleave(Hq // Hkv, dim=0)[None]
        o = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
        outs.append(o[0].transpose(0, 1).reshape(b - a, Hq * D))
    O = torch.cat(outs)
    O.backward(torch.tensor(dO))
    lse = attention_lse(shape, cu, Q, K)
    dQ, dK, dV = attention_backward(shape, cu, Q, K, V, O.detach().numpy(), lse, dO)
    for mine, ref in ((dQ, tq.grad), (dK, tk.grad), (dV, tv.grad)):
        assert np.max(np.abs(mine - ref.numpy())) <= 1e-12 * max(1.0, ref.abs().max().item())


def test_softmax_gradient_rows_sum_to_zero():
    # adding one vector to every key of a sequence leaves the softmax unchanged, so
    # for a consistent record the key gradients of each (sequence, kv head) sum to 0
    shape, cu, T, W, X, R = make(11)
    _, rec = layer_forward(shape, cu, None, X, W)
    dO = np.random.default_rng(12).normal(0, 1, rec["O"].shape)
    dQ, dK, dV = attention_backward(shape, cu, rec["Q"], rec["K"], rec["V"], rec["O"], rec["LSE"], dO)
    D = shape.head_dim
    for s in range(len(cu) - 1):
        blk = dK[cu[s]:cu[s + 1]].reshape(-1, shape.n_kv_heads, D)
        # sum_j dK_j = sum_i (sum_j ds_ij) q_i, and every inner sum is 0
        assert np.max(np.abs(blk.sum(axis=0))) <= 1e-12 * max(1.0, np.abs(blk).max())
    # first token of every sequence attends only to itself (p = 1) => dQ = 0
    for s in range(len(cu) - 1):
        assert np.max(np.abs(dQ[cu[s]])) <= 1e-13
    # single-token sequence: attention is the identity on V
    a = int(cu[0])
    G = shape.n_q_heads // shape.n_kv_heads
    want = dO[a].reshape(shape.n_kv_heads, G, shape.head_dim).sum(axis=1).reshape(-1)
    assert np.allclose(dV[a], want, atol=1e-13)
    assert np.max(np.abs(dK[a])) <= 1e-13


def test_length_one_sequences_have_no_qk_gradient():
    shape, cu, T, W, X, R = make(13, lens=(1, 1, 1, 1))
    _, rec = layer_forward(shape, cu, None, X, W)
    g = layer_backward_reuse(shape, cu, None, rec, W, R)
    assert np.max(np.abs(g["dWq"])) <= 1e-13 and np.max(np.abs(g["dWk"])) <= 1e-13
    assert np.max(np.abs(g["dWv"])) > 1e-3


def test_rope_is_orthogonal_and_identity_at_position_zero():
    rng = np.random.default_rng(0)
    x = rng.normal(0, 1, (6, 3, 8))
    pos = np.array([0, 1, 2, 17, 100, 4095], dtype=np.float64)
    y = _rope(x, pos, 10000.0, +1)
    assert np.array_equal(y[0], x[0])
    half = 4
    n_in = x[..., :half] ** 2 + x[..., half:] ** 2
    n_out = y[..., :half] ** 2 + y[..., half:] ** 2
    assert np.allclose(n_in, n_out, rtol=1e-13)
    assert np.allclose(_rope(y, pos, 10000.0, -1), x, atol=1e-12)
    # textbook value: pair 0 has theta = 1, so position p rotates (1, 0) to (cos p, sin p)
    e = np.zeros((1, 1, 8)); e[0, 0, 0] = 1.0
    r = _rope(e, np.array([2.0]), 10000.0, +1)
    assert np.isclose(r[0, 0, 0], np.cos(2.0)) and np.isclose(r[0, 0, 4], np.sin(2.0))
    # pair i uses base^(-2i/D)
    e = np.zeros((1, 1, 8)); e[0, 0, 1] = 1.0
    r = _rope(e, np.array([3.0]), 10000.0, +1)
    assert np.isclose(r[0, 0, 5], np.sin(3.0 * 10000.0 ** (-2.0 / 8)))


def test_rmsnorm_backward_closed_form():
    rng = np.random.default_rng(1)
    x, g, dh = rng.normal(0, 1, (5, 12)), 1 + rng.normal(0, 0.1, 12), rng.normal(0, 1, (5, 12))
    for eps in (1e-2, 1e-6):
        h, r = _rms_norm(x, g, eps)
        assert np.allclose(np.mean((h / g) ** 2, axis=1), 1 - eps * r[:, 0] ** 2)
        dx, dg = _rms_norm_backward(dh, x, g, r)
        # <x, dx> = eps * r^3 * sum(g * dh * x): the gradient is orthogonal to x as eps -> 0
        lhs = np.sum(x * dx, axis=1)
        rhs = eps * r[:, 0] ** 3 * np.sum(g * dh * x, axis=1)
        assert np.allclose(lhs, rhs, rtol=1e-9, atol=1e-14)


def test_special_cases():
    shape, cu, T, W, X, R = make(21)
    _, rec = layer_forward(shape, cu, None, X, W)
    g = layer_backward_reuse(shape, cu, None, rec, W, R)
    # linear in dY
    g3 = layer_backward_reuse(shape, cu, None, rec, W, 3.0 * R)
    for k in GRADS:
        assert np.max(np.abs(g3[k] - 3.0 * g[k])) <= 1e-12 * np.abs(g3[k]).max()
    # Wd = 0: no gradient reaches the MLP weights or flows through the MLP
    W0 = dict(W, Wd=np.zeros_like(W["Wd"]))
    _, rec0 = layer_forward(shape, cu, None, X, W0)
    g0 = layer_backward_reuse(shape, cu, None, rec0, W0, R)
    assert np.max(np.abs(g0["dWg"])) == 0 and np.max(np.abs(g0["dWu"])) == 0 and np.max(np.abs(g0["dg2"])) == 0
    # Wo = 0 and Wd = 0: the layer is the identity, dX = dY
    W00 = dict(W0, Wo=np.zeros_like(W["Wo"]))
    _, rec00 = layer_forward(shape, cu, None, X, W00)
    g00 = layer_backward_reuse(shape, cu, None, rec00, W00, R)
    assert np.array_equal(g00["dX"], R)
    # loss mask == zeroed dY rows, bit for bit
    mask = (np.random.default_rng(2).random(T) < 0.5).astype(np.uint8)
    Rz = R.copy(); Rz[mask == 0] = 0
    gm = layer_backward_reuse(shape, cu, None, rec, W, R, loss_mask=mask)
    gz = layer_backward_reuse(shape, cu, None, rec, W, Rz)
    for k in GRADS:
        assert np.array_equal(gm[k], gz[k])


def test_identical_query_heads_in_a_group_scale_key_gradient():
    D, n, G = 8, 6, 3
    rng = np.random.default_rng(5)
    cu = np.array([0, n])
    q1, K, V, dO1 = rng.normal(0, 1, (n, D)), rng.normal(0, 1, (n, D)), rng.normal(0, 1, (n, D)), rng.normal(0, 1, (n, D))
    s1 = LayerShape(8, 1, 1, D, 8)
    lse1 = attention_lse(s1, cu, q1, K)
    P = np.exp(np.where(np.tril(np.ones((n, n), bool)), q1 @ K.T / np.sqrt(D) - lse1, -np.inf))
    O1 = P @ V
    dQ1, dK1, dV1 = attention_backward(s1, cu, q1, K, V, O1, lse1, dO1)
    sG = LayerShape(8, G, 1, D, 8)
    rep = lambda a: np.tile(a, (1, G))
    dQG, dKG, dVG = attention_backward(sG, cu, rep(q1), K, V, rep(O1), np.tile(lse1, (1, G)), rep(dO1))
    assert np.allclose(dKG, G * dK1, rtol=1e-12) and np.allclose(dVG, G * dV1, rtol=1e-12)
    assert np.allclose(dQG, rep(dQ1), rtol=1e-12)


@pytest.mark.parametrize("m", [1, 3, 8])
def test_tail_rows_shortcut_equals_full_backward(m):
    # the sampled-row helper used at full size is the same function as the full oracle
    shape, cu, T, W, X, R = make(31, lens=(4, 9))
    _, rec = layer_forward(shape, cu, None, X, W)
    rec = {k: v + 0.01 * np.random.default_rng(1).normal(0, 1, v.shape) for k, v in rec.items()}  # any record
    full = layer_backward_reuse(shape, cu, None, rec, W, R)["dX"]
    for s in range(2):
        a, b = int(cu[s]), int(cu[s + 1])
        mm = min(m, b - a)
        seq = {k: rec[k][a:b] for k in RECORD_KEYS}
        tail = layer_backward_reuse_tail_rows(shape, None, seq, W, R[b - mm:b])
        assert np.max(np.abs(tail - full[b - mm:b])) <= 1e-12 * np.abs(full).max()


def test_complete_record_restores_the_dropped_tensors():
    # a forward's record with X2, O, LSE dropped is completed to the same record (Section 4.3.2: a saved
    # tensor may be recomputed instead of loaded); tensors that are present are passed through untouched
    from oracle import complete_record
    shape, cu, T, W, X, R = make(21, Hq=6, Hkv=2, D=4, F=20, lens=(3, 1, 0, 6))
    _, rec = layer_forward(shape, cu, None, X, W)
    six = {k: rec[k] for k in ("X", "Q", "K", "V", "G", "U")}
    full = complete_record(shape, cu, six, W)
    for k in RECORD_KEYS:
        np.testing.assert_allclose(full[k], rec[k], rtol=1e-12, atol=1e-12, err_msg=k)
    # layer input, query and KV cache alone: the MLP pre-activations come back too
    four = complete_record(shape, cu, {k: rec[k] for k in ("X", "Q", "K", "V")}, W)
    for k in RECORD_KEYS:
        np.testing.assert_allclose(four[k], rec[k], rtol=1e-12, atol=1e-12, err_msg=k)
    # a wrong gain or a swapped gate/up weight is visible: the completed tensors differ from the forward's
    swapped = complete_record(shape, cu, {k: rec[k] for k in ("X", "Q", "K", "V")}, dict(W, Wg=W["Wu"], Wu=W["Wg"]))
    assert np.max(np.abs(swapped["G"] - rec["G"])) > 1e-3
    marked = dict(six, X2=rec["X2"] + 1.0)
    assert np.array_equal(complete_record(shape, cu, marked, W)["X2"], rec["X2"] + 1.0)
    g_full = layer_backward_reuse(shape, cu, None, rec, W, R)
    g_six = layer_backward_reuse(shape, cu, None, full, W, R)
    for k in g_full:
        np.testing.assert_allclose(g_six[k], g_full[k], rtol=1e-10, atol=1e-12, err_msg=k)
