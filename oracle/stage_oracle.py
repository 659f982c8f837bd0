"""CPU oracle for one pipeline stage's decoder-block stack.  TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this file.  It shares no code with the HIP library and never calls it.

What it defines.  The paper (System Model and Terminology, Table 1) takes a
*stage* to be a run of consecutive layers of a GPT- or Llama-family model
(Evaluation, Table 2) held on one GPU; an inference task is forward-only, a
training task is forward plus backward; decoding extends a prefilled context
(Autoregressive Generation).  The paper does not spell out the block
arithmetic, so the textbook pre-LayerNorm GPT block and the RMSNorm + RoPE +
SwiGLU LLaMA block are written out below as plain definitions:

  * dense matmuls (numpy's matmul is the only library primitive used),
  * a fully materialised score matrix with an explicit causal mask,
  * two-pass max-subtracted softmax,
  * contiguous per-request K/V arrays (no pages),
  * every intermediate kept, backward by the hand-derived chain rule.

Everything is computed in the dtype of the arrays passed in (float64 in the
parity tests; float32 works too).  No blocking, fusion or reordering.

Parameters arrive as one flat vector in boundary order; every linear is
[out, in] row-major:
  GPT block  : ln1_g ln1_b W_qkv[3d,d] b_qkv W_o[d,d] b_o ln2_g ln2_b
               W_1[F,d] b_1 W_2[d,F] b_2
  LLaMA block: g1 W_qkv[3d,d] W_o[d,d] g2 W_gu[2F,d] (gate rows then up rows)
               W_d[d,F]

Pins (tests/test_oracle_pins.py): central finite differences of every
gradient, cached decode == full causal recompute, chunked prefill == single
prefill, causal invariance, softmax/LN/RMSNorm/RoPE closed forms, attention
special cases, linearity of the backward in dY, identity stage when the
branch output matrices are zero, independent brute-force loops on tiny shapes.
Large shapes have no pin of their own: the code is shape-generic.
"""
from __future__ import annotations

import math

import numpy as np

# --------------------------------------------------------------------------
# parameter slicing (the oracle's own copy of the boundary order)
# --------------------------------------------------------------------------


def _layer_fields(cfg):
    d, F = cfg["d_model"], cfg["d_ff"]
    if cfg["block"] == "gpt":
        return [("ln1_g", (d,)), ("ln1_b", (d,)), ("W_qkv", (3 * d, d)), ("b_qkv", (3 * d,)),
                ("W_o", (d, d)), ("b_o", (d,)), ("ln2_g", (d,)), ("ln2_b", (d,)),
                ("W_1", (F, d)), ("b_1", (F,)), ("W_2", (d, F)), ("b_2", (d,))]
    return [("g1", (d,)), ("W_qkv", (3 * d, d)), ("W_o", (d, d)), ("g2", (d,)),
            ("W_gu", (2 * F, d)), ("W_d", (d, F))]


def split_params(cfg, flat):
    """Flat vector -> list (one per block) of dicts of views."""
    layers, off = [], 0
    for _ in range(cfg["n_layers"]):
        p = {}
        for name, shape in _layer_fields(cfg):
            n = int(np.prod(shape))
            p[name] = flat[off:off + n].reshape(shape)
            off += n
        layers.append(p)
    assert off == flat.size, "parameter vector has the wrong length"
    return layers


def n_params(cfg):
    return cfg["n_layers"] * sum(int(np.prod(s)) for _, s in _layer_fields(cfg))


# --------------------------------------------------------------------------
# elementwise pieces
# --------------------------------------------------------------------------


def layer_norm(x, gamma, beta, eps):
    """(x - mean) / sqrt(var + eps) * gamma + beta, biased variance over the last axis."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    r = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * r
    return xhat * gamma + beta, xhat, r


def layer_norm_bwd(dh, xhat, r, gamma):
    dxhat = dh * gamma
    dx = r * (dxhat - dxhat.mean(axis=-1, keepdims=True)
              - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, (dh * xhat).sum(axis=0), dh.sum(axis=0)


def rms_norm(x, g, eps):
    """x / sqrt(mean(x^2) + eps) * g."""
    r = 1.0 / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps)
    xhat = x * r
    return xhat * g, xhat, r


def rms_norm_bwd(dh, xhat, r, g):
    dxhat = dh * g
    dx = r * (dxhat - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, (dh * xhat).sum(axis=0)


_C_GELU = math.sqrt(2.0 / math.pi)


def _erf(x):
    return np.vectorize(math.erf, otypes=[x.dtype])(x)


def gelu(u, kind):
    if kind == "gelu_tanh":
        return 0.5 * u * (1.0 + np.tanh(_C_GELU * (u + 0.044715 * u ** 3)))
    return 0.5 * u * (1.0 + _erf(u / math.sqrt(2.0)))


def gelu_grad(u, kind):
    if kind == "gelu_tanh":
        t = np.tanh(_C_GELU * (u + 0.044715 * u ** 3))
        return 0.5 * (1.0 + t) + 0.5 * u * (1.0 - t * t) * _C_GELU * (1.0 + 3.0 * 0.044715 * u * u)
    Phi = 0.5 * (1.0 + _erf(u / math.sqrt(2.0)))
    phi = np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)
    return Phi + u * phi


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def silu(z):
    return z * sigmoid(z)


def rope_angles(pos, head_dim, theta, dtype):
    """angle[t, i] = pos[t] * theta^(-2 i / head_dim), i < head_dim / 2."""
    i = np.arange(head_dim // 2, dtype=dtype)
    inv = np.asarray(theta, dtype) ** (-2.0 * i / head_dim)
    return np.asarray(pos, dtype)[:, None] * inv[None, :]


def rope(x, pos, theta, sign=1.0):
    """Half-split rotary embedding on x[T, h, dh]: the pair (x_i, x_{i+dh/2})
    is rotated by angle[t, i]; sign=-1 rotates back (the transpose, used for
    gradients)."""
    T, h, dh = x.shape
    ang = rope_angles(pos, dh, theta, x.dtype) * sign
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., : dh // 2], x[..., dh // 2:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


# --------------------------------------------------------------------------
# attention on one sequence: queries at absolute positions past .. past+Lq-1
# attend to keys 0 .. past+i
# --------------------------------------------------------------------------


def attention_probs(q, k, past):
    """q[Lq, dh], k[Lk, dh] (Lk = past + Lq) -> P[Lq, Lk], masked entries exactly 0."""
    Lq, dh = q.shape
    Lk = k.shape[0]
    s = (q @ k.T) / math.sqrt(dh)
    allowed = np.arange(Lk)[None, :] <= (past + np.arange(Lq))[:, None]
    s = np.where(allowed, s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    e = np.where(allowed, np.exp(s - m), 0.0)
    return e / e.sum(axis=1, keepdims=True)


def attention(q, k, v, past):
    """q[Lq,h,dh], k,v[Lk,h,dh] -> o[Lq,h,dh], P[h,Lq,Lk]."""
    Lq, h, dh = q.shape
    o = np.empty_like(q)
    P = np.empty((h, Lq, k.shape[0]), q.dtype)
    for j in range(h):
        P[j] = attention_probs(q[:, j], k[:, j], past)
        o[:, j] = P[j] @ v[:, j]
    return o, P


def attention_bwd(do, q, k, v, P):
    """Gradients of attention() for past = 0 (training)."""
    Lq, h, dh = q.shape
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    sc = 1.0 / math.sqrt(dh)
    for j in range(h):
        p = P[j]
        dv[:, j] = p.T @ do[:, j]
        dp = do[:, j] @ v[:, j].T
        ds = p * (dp - (dp * p).sum(axis=1, keepdims=True))
        dq[:, j] = (ds @ k[:, j]) * sc
        dk[:, j] = (ds.T @ q[:, j]) * sc
    return dq, dk, dv


# --------------------------------------------------------------------------
# one block, forward over a list of sequences that share the weights
# --------------------------------------------------------------------------


def _norm1(cfg, p, x):
    if cfg["block"] == "gpt":
        return layer_norm(x, p["ln1_g"], p["ln1_b"], cfg["norm_eps"])
    return rms_norm(x, p["g1"], cfg["norm_eps"])


def _norm2(cfg, p, x):
    if cfg["block"] == "gpt":
        return layer_norm(x, p["ln2_g"], p["ln2_b"], cfg["norm_eps"])
    return rms_norm(x, p["g2"], cfg["norm_eps"])


def block_forward(cfg, p, x, pos, k_past=None, v_past=None):
    """One block on one sequence chunk.

    x[Lq, d]; pos[Lq] absolute positions (= past + arange(Lq)); k_past/v_past
    [past, h, dh] or None.  Returns (y, k_all, v_all, saved) where k_all/v_all
    include the new rows (K after RoPE)."""
    d, h, dh, F = cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["d_ff"]
    gpt = cfg["block"] == "gpt"
    Lq = x.shape[0]
    past = 0 if k_past is None else k_past.shape[0]
    h1, xhat1, r1 = _norm1(cfg, p, x)
    qkv = h1 @ p["W_qkv"].T
    if gpt:
        qkv = qkv + p["b_qkv"]
    q = qkv[:, :d].reshape(Lq, h, dh)
    k = qkv[:, d:2 * d].reshape(Lq, h, dh)
    v = qkv[:, 2 * d:].reshape(Lq, h, dh)
    if not gpt:
        q = rope(q, pos, cfg["rope_theta"])
        k = rope(k, pos, cfg["rope_theta"])
    k_all = k if past == 0 else np.concatenate([k_past, k], axis=0)
    v_all = v if past == 0 else np.concatenate([v_past, v], axis=0)
    o, P = attention(q, k_all, v_all, past)
    o2 = o.reshape(Lq, d)
    x1 = x + o2 @ p["W_o"].T
    if gpt:
        x1 = x1 + p["b_o"]
    h2, xhat2, r2 = _norm2(cfg, p, x1)
    if gpt:
        u = h2 @ p["W_1"].T + p["b_1"]
        a = gelu(u, cfg["act"])
        y = x1 + a @ p["W_2"].T + p["b_2"]
        ffn_saved = dict(u=u)
    else:
        gu = h2 @ p["W_gu"].T
        gate, up = gu[:, :F], gu[:, F:]
        a = silu(gate) * up
        y = x1 + a @ p["W_d"].T
        ffn_saved = dict(gate=gate, up=up)
    saved = dict(xhat1=xhat1, r1=r1, h1=h1, q=q, k=k, v=v, P=P, o=o2,
                 xhat2=xhat2, r2=r2, h2=h2, a=a, pos=pos, **ffn_saved)
    return y, k_all, v_all, saved


def block_backward(cfg, p, s, dy):
    """Chain rule through block_forward (past = 0).  Returns (dx, grads dict)."""
    d, h, dh, F = cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["d_ff"]
    gpt = cfg["block"] == "gpt"
    L = dy.shape[0]
    g = {}
    # y = x1 + a W2^T (+ b2)
    if gpt:
        da = dy @ p["W_2"]
        g["W_2"] = dy.T @ s["a"]
        g["b_2"] = dy.sum(axis=0)
        du = da * gelu_grad(s["u"], cfg["act"])
        dh2 = du @ p["W_1"]
        g["W_1"] = du.T @ s["h2"]
        g["b_1"] = du.sum(axis=0)
        dn, g["ln2_g"], g["ln2_b"] = layer_norm_bwd(dh2, s["xhat2"], s["r2"], p["ln2_g"])
    else:
        da = dy @ p["W_d"]
        g["W_d"] = dy.T @ s["a"]
        sg = sigmoid(s["gate"])
        dup = da * (s["gate"] * sg)
        dgate = da * s["up"] * sg * (1.0 + s["gate"] * (1.0 - sg))
        dgu = np.concatenate([dgate, dup], axis=1)
        dh2 = dgu @ p["W_gu"]
        g["W_gu"] = dgu.T @ s["h2"]
        dn, g["g2"] = rms_norm_bwd(dh2, s["xhat2"], s["r2"], p["g2"])
    dx1 = dy + dn
    # x1 = x + o Wo^T (+ bo)
    do = dx1 @ p["W_o"]
    g["W_o"] = dx1.T @ s["o"]
    if gpt:
        g["b_o"] = dx1.sum(axis=0)
    dq, dk, dv = attention_bwd(do.reshape(L, h, dh), s["q"], s["k"], s["v"], s["P"])
    if not gpt:
        dq = rope(dq, s["pos"], cfg["rope_theta"], sign=-1.0)
        dk = rope(dk, s["pos"], cfg["rope_theta"], sign=-1.0)
    dqkv = np.concatenate([dq.reshape(L, d), dk.reshape(L, d), dv.reshape(L, d)], axis=1)
    dh1 = dqkv @ p["W_qkv"]
    g["W_qkv"] = dqkv.T @ s["h1"]
    if gpt:
        g["b_qkv"] = dqkv.sum(axis=0)
        dn1, g["ln1_g"], g["ln1_b"] = layer_norm_bwd(dh1, s["xhat1"], s["r1"], p["ln1_g"])
    else:
        dn1, g["g1"] = rms_norm_bwd(dh1, s["xhat1"], s["r1"], p["g1"])
    return dx1 + dn1, g


# --------------------------------------------------------------------------
# stage-level calls (mirror the boundary: prefill, decode, train fwd, train bwd)
# --------------------------------------------------------------------------


def new_cache(cfg, n_requests, dtype=np.float64):
    """cache[layer][request] = [K, V], each [ctx, h, dh] (contiguous, starts empty)."""
    h, dh = cfg["n_heads"], cfg["head_dim"]
    return [[[np.zeros((0, h, dh), dtype), np.zeros((0, h, dh), dtype)]
             for _ in range(n_requests)] for _ in range(cfg["n_layers"])]


def stage_prefill(cfg, flat_params, chunks, cache):
    """chunks: list over requests of x[Lc, d].  Each request's chunk starts at
    absolute position len(cache) and attends to its cached keys plus the causal
    part of the chunk; K (after RoPE) and V rows are appended to the cache.
    Returns the list of outputs y[Lc, d]."""
    layers = split_params(cfg, flat_params)
    outs = []
    for b, x in enumerate(chunks):
        past = cache[0][b][0].shape[0]
        pos = past + np.arange(x.shape[0])
        for l, p in enumerate(layers):
            kp, vp = cache[l][b]
            x, k_all, v_all, _ = block_forward(cfg, p, x, pos, kp if past else None,
                                               vp if past else None)
            cache[l][b] = [k_all, v_all]
        outs.append(x)
    return outs


def block_decode(cfg, p, X, cache_l):
    """One block on one new token per request.  The row-wise steps (norms,
    linear maps, activation) are applied to all B rows at once - they do not mix
    rows - and attention runs per request over its own cache, which receives
    the new K (after RoPE) and V row first."""
    d, h, dh, F = cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["d_ff"]
    gpt = cfg["block"] == "gpt"
    B = X.shape[0]
    h1, _, _ = _norm1(cfg, p, X)
    qkv = h1 @ p["W_qkv"].T
    if gpt:
        qkv = qkv + p["b_qkv"]
    o = np.empty((B, d), X.dtype)
    for b in range(B):
        K, V = cache_l[b]
        pos = np.array([K.shape[0]])
        q = qkv[b:b + 1, :d].reshape(1, h, dh)
        k = qkv[b:b + 1, d:2 * d].reshape(1, h, dh)
        v = qkv[b:b + 1, 2 * d:].reshape(1, h, dh)
        if not gpt:
            q = rope(q, pos, cfg["rope_theta"])
            k = rope(k, pos, cfg["rope_theta"])
        K = np.concatenate([K, k], axis=0)
        V = np.concatenate([V, v], axis=0)
        cache_l[b] = [K, V]
        ob, _ = attention(q, K, V, K.shape[0] - 1)
        o[b] = ob.reshape(d)
    x1 = X + o @ p["W_o"].T
    if gpt:
        x1 = x1 + p["b_o"]
    h2, _, _ = _norm2(cfg, p, x1)
    if gpt:
        a = gelu(h2 @ p["W_1"].T + p["b_1"], cfg["act"])
        return x1 + a @ p["W_2"].T + p["b_2"]
    gu = h2 @ p["W_gu"].T
    return x1 + (silu(gu[:, :F]) * gu[:, F:]) @ p["W_d"].T


def stage_decode(cfg, flat_params, X, cache):
    """One new token per request: X[B, d] -> Y[B, d]; request b's token sits at
    position ctx_b = len(cache) and attends over ctx_b + 1 keys."""
    x = X
    for l, p in enumerate(split_params(cfg, flat_params)):
        x = block_decode(cfg, p, x, cache[l])
    return x


def block_forward_rows(cfg, p, x, rows):
    """Rows `rows` of block_forward(cfg, p, x, arange(L))[0] for one sequence
    from position 0, without forming the other output rows: K and V are needed
    for every position, the query side only for the sampled ones."""
    d, h, dh, F = cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["d_ff"]
    gpt = cfg["block"] == "gpt"
    L = x.shape[0]
    rows = np.asarray(rows)
    h1, _, _ = _norm1(cfg, p, x)
    kv = h1 @ p["W_qkv"][d:].T
    q = h1[rows] @ p["W_qkv"][:d].T
    if gpt:
        kv = kv + p["b_qkv"][d:]
        q = q + p["b_qkv"][:d]
    k = kv[:, :d].reshape(L, h, dh)
    v = kv[:, d:].reshape(L, h, dh)
    q = q.reshape(len(rows), h, dh)
    if not gpt:
        k = rope(k, np.arange(L), cfg["rope_theta"])
        q = rope(q, rows, cfg["rope_theta"])
    o = np.empty((len(rows), d), x.dtype)
    for i, t in enumerate(rows):
        ob, _ = attention(q[i:i + 1], k[: t + 1], v[: t + 1], int(t))
        o[i] = ob.reshape(d)
    x1 = x[rows] + o @ p["W_o"].T
    if gpt:
        x1 = x1 + p["b_o"]
    h2, _, _ = _norm2(cfg, p, x1)
    if gpt:
        a = gelu(h2 @ p["W_1"].T + p["b_1"], cfg["act"])
        return x1 + a @ p["W_2"].T + p["b_2"]
    gu = h2 @ p["W_gu"].T
    return x1 + (silu(gu[:, :F]) * gu[:, F:]) @ p["W_d"].T


def stage_train_fwd(cfg, flat_params, X):
    """X[B, L, d] -> (Y[B, L, d], saved).  Each sequence starts at position 0."""
    layers = split_params(cfg, flat_params)
    B, L, d = X.shape
    Y = np.empty_like(X)
    saved = []
    pos = np.arange(L)
    for b in range(B):
        x = X[b]
        per_layer = []
        for p in layers:
            x, _, _, s = block_forward(cfg, p, x, pos)
            per_layer.append(s)
        Y[b] = x
        saved.append(per_layer)
    return Y, saved


def stage_train_bwd(cfg, flat_params, saved, dY):
    """dY[B, L, d] -> (dX[B, L, d], flat parameter gradient summed over all
    tokens of the micro-batch, boundary order)."""
    layers = split_params(cfg, flat_params)
    dflat = np.zeros_like(flat_params)
    dlayers = split_params(cfg, dflat)
    dX = np.empty_like(dY)
    for b in range(dY.shape[0]):
        dx = dY[b]
        for l in range(cfg["n_layers"] - 1, -1, -1):
            dx, g = block_backward(cfg, layers[l], saved[b][l], dx)
            for name, val in g.items():
                dlayers[l][name] += val
        dX[b] = dx
    return dX, dflat


# ---------------------------------------------------------------------------------------
# Model update after a training task (Model Update Synchronization: every co-located
# instance applies its own local updates, so that later inference tasks on the same stage
# are served from the updated weights).  The paper names no optimizer; the two textbook
# rules are written out as plain definitions.
#
#   SGD with momentum and L2 decay:   g' = g + wd w ;  b <- mu b + g' ;  w <- w - lr b
#   AdamW (decoupled weight decay):   m <- b1 m + (1 - b1) g ;  v <- b2 v + (1 - b2) g^2
#                                     w <- w - lr ( m / (1 - b1^t) / (sqrt(v / (1 - b2^t)) + eps) + wd w )
#
# `decay` is a 0/1 array: decay applies to the linear maps' weight matrices only (not to
# normalisation gains or biases).  `g` is first multiplied by grad_scale (e.g. one over the
# number of accumulated micro-batches).  `t` counts steps from 1.
def optimizer_step(kind, w, g, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0,
                   momentum=0.0, grad_scale=1.0, decay=None):
    """Returns (w, m, v) after one update; inputs are not modified.  For SGD `m` is the
    momentum buffer and `v` passes through unchanged."""
    w = np.array(w, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64) * grad_scale
    m = np.array(m, dtype=np.float64)
    v = np.array(v, dtype=np.float64)
    wd = weight_decay * (np.ones_like(w) if decay is None else np.asarray(decay, dtype=np.float64))
    if kind == "sgd":
        g = g + wd * w
        m = momentum * m + g
        return w - lr * m, m, v
    if kind == "adamw":
        m = beta1 * m + (1.0 - beta1) * g
        v = beta2 * v + (1.0 - beta2) * g * g
        m_hat = m / (1.0 - beta1 ** t)
        v_hat = v / (1.0 - beta2 ** t)
        return w - lr * (m_hat / (np.sqrt(v_hat) + eps) + wd * w), m, v
    raise ValueError(kind)


def decay_mask(cfg):
    """1 for elements of weight matrices (2-D fields), 0 for gains and biases, in boundary order."""
    out = np.zeros(n_params(cfg))
    off = 0
    for _ in range(cfg["n_layers"]):
        for _name, shape in _layer_fields(cfg):
            n = int(np.prod(shape))
            if len(shape) == 2:
                out[off:off + n] = 1.0
            off += n
    return out
