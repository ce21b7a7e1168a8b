"""Oracle for one pre-norm decoder layer: forward, and backward from saved activations.

Test infrastructure only (see the package docstring).  All arithmetic is float64.

Paper basis: Section 1 / Section 2.5.1 (the activations saved while serving equal
the ones a training forward would recompute, so the backward pass may consume
them directly), Section 4.1 (what is saved: the per-layer activations and the KV
cache of the prompt tokens), Section 4.2 / 4.3.2 (backward runs per layer).  The
paper prints no equations; the layer is the Llama-family decoder layer it trains
(Section 6): y = x2 + W_d (silu(W_g h2) * (W_u h2)), h2 = RMSNorm(x2; g2),
x2 = x + W_o Attn(RoPE(W_q h1), RoPE(W_k h1), W_v h1), h1 = RMSNorm(x; g1).

Conventions (readings taken where the paper is silent):
  * weights are [out, in] row-major, y = x W^T;
  * RMSNorm: x * (mean(x^2) + eps)^(-1/2) * g, eps inside the root;
  * RoPE pairs element i with i + D/2, angle = position * base^(-2i/D);
  * query head h reads KV head h // (Hq // Hkv); softmax scale 1/sqrt(D);
    token i attends to tokens j <= i of its own sequence, masked terms are
    exactly absent;
  * the saved record is {X, X2, Q, K, V, O, LSE, G, U}: Q and K after RoPE (what a
    KV cache holds), G and U before the activation, LSE the natural-log
    normaliser of each (token, query head) softmax row.
"""
from dataclasses import dataclass
import numpy as np

RECORD_KEYS = ("X", "X2", "Q", "K", "V", "O", "LSE", "G", "U")
WEIGHT_KEYS = ("Wq", "Wk", "Wv", "Wo", "Wg", "Wu", "Wd", "g1", "g2")


@dataclass
class LayerShape:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    rms_eps: float = 1e-6
    rope_base: float = 10000.0


def _positions(cu, positions, T):
    if positions is not None:
        return np.asarray(positions, dtype=np.float64)
    pos = np.zeros(T, dtype=np.float64)
    for s in range(len(cu) - 1):
        pos[cu[s]:cu[s + 1]] = np.arange(cu[s + 1] - cu[s])
    return pos


def _rms_norm(x, g, eps):
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return x * r * g, r


def _rms_norm_backward(dh, x, g, r):
    """Gradient of h = x * r * g with r = (mean(x^2)+eps)^(-1/2).  Returns (dx, dg)."""
    n = x.shape[-1]
    gd = g * dh
    dx = r * gd - x * (r ** 3) / n * np.sum(gd * x, axis=-1, keepdims=True)
    dg = np.sum(dh * x * r, axis=0)
    return dx, dg


def _rope(x, pos, base, sign):
    """x: [T, heads, D].  sign=+1 rotates by +angle (forward), -1 by -angle (the
    transpose of the forward rotation, i.e. its gradient map)."""
    D = x.shape[-1]
    half = D // 2
    theta = base ** (-2.0 * np.arange(half, dtype=np.float64) / D)
    a = pos[:, None] * theta[None, :]
    c, s = np.cos(a)[:, None, :], np.sin(a)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - sign * x2 * s, x2 * c + sign * x1 * s], axis=-1)


def _sigmoid(g):
    return 1.0 / (1.0 + np.exp(-g))


def attention_lse(shape, cu_seqlens, Q, K):
    """LSE[t, h] = log sum_{j<=t, same sequence} exp(Q[t,h] . K[j, h//G] / sqrt(D))."""
    T = Q.shape[0]
    Hq, Hkv, D = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    G = Hq // Hkv
    Qh, Kh = Q.reshape(T, Hq, D), K.reshape(T, Hkv, D)
    lse = np.zeros((T, Hq), dtype=np.float64)
    for s in range(len(cu_seqlens) - 1):
        a, b = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        n = b - a
        if n == 0:
            continue
        allowed = np.tril(np.ones((n, n), dtype=bool))
        for h in range(Hq):
            sc = Qh[a:b, h] @ Kh[a:b, h // G].T / np.sqrt(D)
            sc = np.where(allowed, sc, -np.inf)
            m = sc.max(axis=1, keepdims=True)
            lse[a:b, h] = (m + np.log(np.sum(np.exp(sc - m), axis=1, keepdims=True)))[:, 0]
    return lse


def layer_forward(shape, cu_seqlens, positions, X, W):
    """Returns (Y [T,H], record dict with RECORD_KEYS)."""
    X = np.asarray(X, dtype=np.float64)
    T, H = X.shape
    Hq, Hkv, D = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    G = Hq // Hkv
    pos = _positions(cu_seqlens, positions, T)

    H1, _ = _rms_norm(X, W["g1"], shape.rms_eps)
    Q = _rope((H1 @ W["Wq"].T).reshape(T, Hq, D), pos, shape.rope_base, +1)
    K = _rope((H1 @ W["Wk"].T).reshape(T, Hkv, D), pos, shape.rope_base, +1)
    V = (H1 @ W["Wv"].T).reshape(T, Hkv, D)

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

    X2 = X + O @ W["Wo"].T
    H2, _ = _rms_norm(X2, W["g2"], shape.rms_eps)
    Gt = H2 @ W["Wg"].T
    U = H2 @ W["Wu"].T
    Act = Gt * _sigmoid(Gt) * U
    Y = X2 + Act @ W["Wd"].T
    rec = dict(X=X, X2=X2, Q=Q.reshape(T, Hq * D), K=K.reshape(T, Hkv * D),
               V=V.reshape(T, Hkv * D), O=O, LSE=LSE, G=Gt, U=U)
    return Y, rec


def attention_backward(shape, cu_seqlens, Q, K, V, O, LSE, dO):
    """Gradient of causal grouped-query attention w.r.t. (post-RoPE) Q, K and V,
    from saved Q, K, V, O, LSE and the incoming dO.  Explicit n x n probabilities
    per (sequence, query head); K/V gradients are summed over the query heads that
    share a KV head.  Returns (dQ [T,Hq*D], dK [T,Hkv*D], dV [T,Hkv*D])."""
    T = Q.shape[0]
    Hq, Hkv, D = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    G = Hq // Hkv
    Qh, Kh, Vh = Q.reshape(T, Hq, D), K.reshape(T, Hkv, D), V.reshape(T, Hkv, D)
    Oh, dOh = O.reshape(T, Hq, D), dO.reshape(T, Hq, D)
    delta = np.sum(dOh * Oh, axis=-1)                      # [T, Hq]
    dQ = np.zeros_like(Qh)
    dK = np.zeros_like(Kh)
    dV = np.zeros_like(Vh)
    scale = 1.0 / np.sqrt(D)
    for s in range(len(cu_seqlens) - 1):
        a, b = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        n = b - a
        if n == 0:
            continue
        allowed = np.tril(np.ones((n, n), dtype=bool))
        for h in range(Hq):
            kv = h // G
            sc = Qh[a:b, h] @ Kh[a:b, kv].T * scale
            P = np.where(allowed, np.exp(sc - LSE[a:b, h][:, None]), 0.0)
            dV[a:b, kv] += P.T @ dOh[a:b, h]
            dP = dOh[a:b, h] @ Vh[a:b, kv].T
            dS = P * (dP - delta[a:b, h][:, None])
            dQ[a:b, h] = dS @ Kh[a:b, kv] * scale
            dK[a:b, kv] += dS.T @ Qh[a:b, h] * scale
    return dQ.reshape(T, Hq * D), dK.reshape(T, Hkv * D), dV.reshape(T, Hkv * D)


def layer_backward_reuse(shape, cu_seqlens, positions, rec, W, dY, loss_mask=None):
    """Backward of layer_forward driven ONLY by the saved record `rec`.

    Every record tensor is consumed as given (probabilities from saved Q, K, LSE;
    the softmax-gradient row term from saved O; normalised inputs from saved X and
    X2; the MLP activation from saved G, U), so the result is defined even for a
    record that no forward produced.  loss_mask (uint8 [T] or None): rows of dY
    whose mask is 0 are treated as zero.

    Returns dict: dX and dWq,dWk,dWv,dWo,dWg,dWu,dWd,dg1,dg2.
    """
    X, X2, Q, K, V, O, LSE, Gt, U = (np.asarray(rec[k], dtype=np.float64) for k in RECORD_KEYS)
    T, H = X.shape
    Hq, Hkv, D = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    G = Hq // Hkv
    pos = _positions(cu_seqlens, positions, T)
    dY = np.array(dY, dtype=np.float64)
    if loss_mask is not None:
        dY[np.asarray(loss_mask) == 0] = 0.0

    # MLP: y = x2 + (silu(G) * U) Wd^T
    sig = _sigmoid(Gt)
    Act = Gt * sig * U
    dAct = dY @ W["Wd"]
    dWd = dY.T @ Act
    dG = dAct * U * sig * (1.0 + Gt * (1.0 - sig))
    dU = dAct * Gt * sig
    dH2 = dG @ W["Wg"] + dU @ W["Wu"]
    H2, r2 = _rms_norm(X2, W["g2"], shape.rms_eps)
    dWg = dG.T @ H2
    dWu = dU.T @ H2
    dX2n, dg2 = _rms_norm_backward(dH2, X2, W["g2"], r2)
    dX2 = dY + dX2n

    # attention output projection: x2 = x + O Wo^T
    dO = dX2 @ W["Wo"]
    dWo = dX2.T @ O

    # causal grouped-query attention
    dQ, dK, dV = attention_backward(shape, cu_seqlens, Q, K, V, O, LSE, dO)
    dQ, dK, dV = dQ.reshape(T, Hq, D), dK.reshape(T, Hkv, D), dV.reshape(T, Hkv, D)

    # RoPE backward (rotation by the negative angle), then the QKV projections
    dQp = _rope(dQ, pos, shape.rope_base, -1).reshape(T, Hq * D)
    dKp = _rope(dK, pos, shape.rope_base, -1).reshape(T, Hkv * D)
    dVp = dV.reshape(T, Hkv * D)
    dH1 = dQp @ W["Wq"] + dKp @ W["Wk"] + dVp @ W["Wv"]
    H1, r1 = _rms_norm(X, W["g1"], shape.rms_eps)
    dWq = dQp.T @ H1
    dWk = dKp.T @ H1
    dWv = dVp.T @ H1
    dXn, dg1 = _rms_norm_backward(dH1, X, W["g1"], r1)
    dX = dX2 + dXn
    return dict(dX=dX, dWq=dWq, dWk=dWk, dWv=dWv, dWo=dWo, dWg=dWg, dWu=dWu, dWd=dWd,
                dg1=dg1, dg2=dg2)


def complete_record(shape, cu_seqlens, rec, W):
    """The six-tensor record {X, Q, K, V, G, U} (the tensors the capture step is asked to pack in
    the paper's setting, Section 4.1 / Section 5: layer input, KV cache, query, MLP pre-activations)
    completed to the full record: O and LSE by running causal grouped-query attention on the saved
    post-RoPE Q, K, V, then X2 = X + O Wo^T.  The four-tensor record {X, Q, K, V} (layer input, query and
    KV cache alone) is completed further: G = H2 Wg^T, U = H2 Wu^T with H2 the RMS-normalised X2 under gain
    g2, the forward's own definition of the MLP pre-activations.  Tensors already present in `rec` are kept
    as given.  (The decision between loading a saved tensor and recomputing it is the hedging of
    Section 4.3.2.)"""
    out = {k: np.asarray(v, dtype=np.float64) for k, v in rec.items() if v is not None}
    T = out["X"].shape[0]
    Hq, Hkv, D = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    G = Hq // Hkv
    if "O" not in out or "LSE" not in out:
        Q, K, V = out["Q"].reshape(T, Hq, D), out["K"].reshape(T, Hkv, D), out["V"].reshape(T, Hkv, D)
        LSE = attention_lse(shape, cu_seqlens, out["Q"], out["K"])
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
        out["O"], out["LSE"] = O.reshape(T, Hq * D), LSE
    if "X2" not in out:
        out["X2"] = out["X"] + out["O"] @ np.asarray(W["Wo"], dtype=np.float64).T
    if "G" not in out or "U" not in out:
        H2, _ = _rms_norm(out["X2"], np.asarray(W["g2"], dtype=np.float64), shape.rms_eps)
        if "G" not in out:
            out["G"] = H2 @ np.asarray(W["Wg"], dtype=np.float64).T
        if "U" not in out:
            out["U"] = H2 @ np.asarray(W["Wu"], dtype=np.float64).T
    return out


def layer_backward_recompute(shape, cu_seqlens, positions, X, W, dY, loss_mask=None):
    """The comparison path (Section 6, the separate-cluster baseline): re-run the
    forward from X and the weights, then back-propagate through what it produced."""
    _, rec = layer_forward(shape, cu_seqlens, positions, X, W)
    return layer_backward_reuse(shape, cu_seqlens, positions, rec, W, dY, loss_mask)


def layer_backward_reuse_tail_rows(shape, positions_seq, rec_seq, W, dY_tail):
    """dX rows of the last m tokens of ONE sequence, from the dY rows of those tokens alone.

    Causality makes this exact: the input gradient of token t depends only on output gradients of
    tokens i >= t of the same sequence, so the last m rows of dX need the last m rows of dY and
    nothing else (K and V of all earlier tokens enter through the saved record).  Used to check
    full-size GPU runs on sampled rows; pinned against layer_backward_reuse on small cases.

    rec_seq: record tensors of the one sequence (n tokens); dY_tail: [m, H]; positions_seq: [n] or
    None (0..n-1).  Returns dX_tail [m, H].
    """
    X, X2, Q, K, V, O, LSE, Gt, U = (np.asarray(rec_seq[k], dtype=np.float64) for k in RECORD_KEYS)
    n, H = X.shape
    m = dY_tail.shape[0]
    a = n - m
    Hq, Hkv, D = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    G = Hq // Hkv
    pos = np.arange(n, dtype=np.float64) if positions_seq is None else np.asarray(positions_seq, dtype=np.float64)
    dY = np.asarray(dY_tail, dtype=np.float64)

    sig = _sigmoid(Gt[a:])
    dAct = dY @ W["Wd"]
    dG = dAct * U[a:] * sig * (1.0 + Gt[a:] * (1.0 - sig))
    dU = dAct * Gt[a:] * sig
    dH2 = dG @ W["Wg"] + dU @ W["Wu"]
    _, r2 = _rms_norm(X2[a:], W["g2"], shape.rms_eps)
    dX2n, _ = _rms_norm_backward(dH2, X2[a:], W["g2"], r2)
    dX2 = dY + dX2n
    dO = (dX2 @ W["Wo"]).reshape(m, Hq, D)

    Qh, Kh, Vh, Oh = Q.reshape(n, Hq, D), K.reshape(n, Hkv, D), V.reshape(n, Hkv, D), O.reshape(n, Hq, D)
    delta = np.sum(dO * Oh[a:], axis=-1)
    dQ = np.zeros((m, Hq, D))
    dK = np.zeros((m, Hkv, D))
    dV = np.zeros((m, Hkv, D))
    scale = 1.0 / np.sqrt(D)
    # query rows a..n-1 against all keys 0..n-1; key j is visible to query i iff j <= i
    allowed = np.arange(n)[None, :] <= (a + np.arange(m))[:, None]
    for h in range(Hq):
        kv = h // G
        sc = Qh[a:, h] @ Kh[:, kv].T * scale
        P = np.where(allowed, np.exp(sc - LSE[a:, h][:, None]), 0.0)
        dP = dO[:, h] @ Vh[:, kv].T
        dS = P * (dP - delta[:, h][:, None])
        dQ[:, h] = dS @ Kh[:, kv] * scale
        # keys in the tail receive gradient only from tail queries
        dK[:, kv] += dS[:, a:].T @ Qh[a:, h] * scale
        dV[:, kv] += P[:, a:].T @ dO[:, h]
    dQp = _rope(dQ, pos[a:], shape.rope_base, -1).reshape(m, Hq * D)
    dKp = _rope(dK, pos[a:], shape.rope_base, -1).reshape(m, Hkv * D)
    dH1 = dQp @ W["Wq"] + dKp @ W["Wk"] + dV.reshape(m, Hkv * D) @ W["Wv"]
    _, r1 = _rms_norm(X[a:], W["g1"], shape.rms_eps)
    dXn, _ = _rms_norm_backward(dH1, X[a:], W["g1"], r1)
    return dX2 + dXn
