"""What 16-bit *storage* alone costs: the stage in float64 arithmetic with one rounding hook on every tensor
that the GPU path keeps in 16 bits between kernels.  TEST INFRASTRUCTURE, derived from the oracle's pieces
(norms, rotary embedding, activations come from oracle/stage_oracle.py; nothing here is shared with the HIP
library).

Purpose: the bar for a stage run with bf16 matrix-core operands.  bf16 keeps 8 significant bits, so every
stored activation and gradient carries a relative rounding of up to 2^-9; a weight gradient dW = dz^T a sums
T products of two such tensors, each of which was itself computed from rounded tensors.  This model applies
exactly those roundings and nothing else (exact products, exact sums), so its distance from the oracle is the
error that any implementation with that storage format has, however it computes.  With `names` restricted to
one tensor it answers which stored tensor matters (none stands out: see tests/test_storage_rounding_model.py).

Tensor names (the stage's buffers): h1, qkv0 (the projection's 16-bit result before the rotary embedding,
only where the rotation is a pass of its own), qkv (q and k after the rotation, v), P (softmax probabilities
as the second attention product reads them), o, h2, up (FFN pre-activation), act; backward: g16 (the 16-bit
copy of the residual-stream gradient), dact, dup, dh2, d_o, dS, dqkv, dh1.
"""
import math

import numpy as np
import torch

from oracle import stage_oracle as O
from paper_2507_21276_amd import synth_inputs as S

NAMES = ["h1", "qkv0", "qkv", "P", "o", "h2", "up", "act", "g16", "dact", "dup", "dh2", "d_o", "dS", "dqkv", "dh1"]


def round_bf16(x):
    return torch.from_numpy(np.ascontiguousarray(x, np.float64)).to(torch.bfloat16).to(torch.float64).numpy()


def round_f16(x):
    # torch's conversion (threaded; 20x numpy's) goes through float32: a double rounding that moves a value by
    # one more fp16 ulp about once in 2^13 elements, which a model of rounding noise does not notice
    return torch.from_numpy(np.ascontiguousarray(x, np.float64)).to(torch.float16).to(torch.float64).numpy()


def train(cfg, flat, X, dY, names, rnd, grad_scale=1.0):
    """(Y, dX, dParams) of one training task with the tensors in `names` rounded by `rnd` where they are stored.
    grad_scale: the power of two the backward pass multiplies the gradient stream by on entry (results are
    divided by it), as the stage does to keep small gradients in the normal range of fp16."""
    r = (lambda n, x: rnd(x) if n in names else x)
    gpt = cfg["block"] == "gpt"
    layers = O.split_params(cfg, flat)
    d, h, dh, F = cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["d_ff"]
    B, L, _ = X.shape
    pos = np.arange(L)
    allowed = np.arange(L)[None, :] <= np.arange(L)[:, None]
    dflat = np.zeros_like(flat)
    dl = O.split_params(cfg, dflat)
    Y, dX = np.empty_like(X), np.empty_like(X)
    sc = 1.0 / math.sqrt(dh)
    norm = (lambda x, p, i: O.layer_norm(x, p[f"ln{i}_g"], p[f"ln{i}_b"], cfg["norm_eps"])) if gpt else \
           (lambda x, p, i: O.rms_norm(x, p[f"g{i}"], cfg["norm_eps"]))
    for b in range(B):
        x, saved = X[b], []
        for p in layers:
            h1, xhat1, r1 = norm(x, p, 1)
            h1 = r("h1", h1)
            qkv = h1 @ p["W_qkv"].T + (p["b_qkv"] if gpt else 0.0)
            q, k, v = (qkv[:, i * d:(i + 1) * d].reshape(L, h, dh) for i in range(3))
            if not gpt:
                q, k = r("qkv0", q), r("qkv0", k)
                q, k = O.rope(q, pos, cfg["rope_theta"]), O.rope(k, pos, cfg["rope_theta"])
            q, k, v = r("qkv", q), r("qkv", k), r("qkv", v)
            o, lse = np.empty_like(q), np.empty((L, h))
            for j in range(h):
                s = np.where(allowed, (q[:, j] @ k[:, j].T) * sc, -np.inf)
                m = s.max(1, keepdims=True)
                e = np.where(allowed, np.exp(s - m), 0.0)
                o[:, j] = (r("P", e) @ v[:, j]) / e.sum(1, keepdims=True)
                lse[:, j] = (m + np.log(e.sum(1, keepdims=True)))[:, 0]
            o = r("o", o.reshape(L, d))
            x1 = x + o @ p["W_o"].T + (p["b_o"] if gpt else 0.0)
            h2, xhat2, r2 = norm(x1, p, 2)
            h2 = r("h2", h2)
            if gpt:
                up = r("up", h2 @ p["W_1"].T + p["b_1"])
                act = r("act", O.gelu(up, cfg["act"]))
                y = x1 + act @ p["W_2"].T + p["b_2"]
            else:
                up = r("up", h2 @ p["W_gu"].T)
                act = r("act", O.silu(up[:, :F]) * up[:, F:])
                y = x1 + act @ p["W_d"].T
            saved.append(dict(xhat1=xhat1, r1=r1, h1=h1, q=q, k=k, v=v, lse=lse, o=o, xhat2=xhat2, r2=r2, h2=h2,
                              up=up, act=act))
            x = y
        Y[b] = x
        g = dY[b] * grad_scale
        for l in range(cfg["n_layers"] - 1, -1, -1):
            p, s_, gl = layers[l], saved[l], dl[l]
            g16 = r("g16", g)
            w_dn, w_up = ("W_2", "W_1") if gpt else ("W_d", "W_gu")
            dact = r("dact", g16 @ p[w_dn])
            gl[w_dn] += (g16.T @ s_["act"]) / grad_scale
            if gpt:
                gl["b_2"] += g16.sum(0) / grad_scale
                dup = r("dup", dact * O.gelu_grad(s_["up"], cfg["act"]))
                gl["b_1"] += dup.sum(0) / grad_scale
            else:
                gate, upv = s_["up"][:, :F], s_["up"][:, F:]
                sg = O.sigmoid(gate)
                dup = r("dup", np.concatenate([dact * upv * sg * (1.0 + gate * (1.0 - sg)), dact * (gate * sg)], 1))
            dh2 = r("dh2", dup @ p[w_up])
            gl[w_up] += (dup.T @ s_["h2"]) / grad_scale
            if gpt:
                dn, dg, db = O.layer_norm_bwd(dh2, s_["xhat2"], s_["r2"], p["ln2_g"])
                gl["ln2_g"] += dg / grad_scale
                gl["ln2_b"] += db / grad_scale
            else:
                dn, dg = O.rms_norm_bwd(dh2, s_["xhat2"], s_["r2"], p["g2"])
                gl["g2"] += dg / grad_scale
            g1 = g + dn
            g16 = r("g16", g1)
            do = r("d_o", g16 @ p["W_o"]).reshape(L, h, dh)
            gl["W_o"] += (g16.T @ s_["o"]) / grad_scale
            if gpt:
                gl["b_o"] += g16.sum(0) / grad_scale
            dq, dk, dv = (np.empty((L, h, dh)) for _ in range(3))
            o3 = s_["o"].reshape(L, h, dh)
            for j in range(h):
                q, k, v = s_["q"][:, j], s_["k"][:, j], s_["v"][:, j]
                P = np.where(allowed, np.exp(np.where(allowed, (q @ k.T) * sc, -np.inf) - s_["lse"][:, j:j + 1]), 0.0)
                D = (do[:, j] * o3[:, j]).sum(1, keepdims=True)
                dv[:, j] = r("P", P).T @ do[:, j]
                dS = r("dS", P * (do[:, j] @ v.T - D))
                dq[:, j], dk[:, j] = (dS @ k) * sc, (dS.T @ q) * sc
            if not gpt:
                dq, dk = O.rope(dq, pos, cfg["rope_theta"], -1.0), O.rope(dk, pos, cfg["rope_theta"], -1.0)
            dqkv = r("dqkv", np.concatenate([dq.reshape(L, d), dk.reshape(L, d), dv.reshape(L, d)], 1))
            dh1 = r("dh1", dqkv @ p["W_qkv"])
            gl["W_qkv"] += (dqkv.T @ s_["h1"]) / grad_scale
            if gpt:
                gl["b_qkv"] += dqkv.sum(0) / grad_scale
                dn1, dg, db = O.layer_norm_bwd(dh1, s_["xhat1"], s_["r1"], p["ln1_g"])
                gl["ln1_g"] += dg / grad_scale
                gl["ln1_b"] += db / grad_scale
            else:
                dn1, dg = O.rms_norm_bwd(dh1, s_["xhat1"], s_["r1"], p["g1"])
                gl["g1"] += dg / grad_scale
            g = g1 + dn1
        dX[b] = g / grad_scale
    return Y, dX, dflat


def errors(cfg, ref, got):
    """max-abs error over the reference tensor's RMS, per output tensor: Y, dX and every parameter gradient."""
    out = {}
    for nm, a, b in (("Y", ref[0], got[0]), ("dX", ref[1], got[1])):
        out[nm] = float(np.abs(a - b).max() / math.sqrt((a ** 2).mean()))
    for name, off, shape, _ in S.param_layout(cfg):
        n = int(np.prod(shape))
        a, b = ref[2][off:off + n], got[2][off:off + n]
        out[name] = float(np.abs(a - b).max() / max(math.sqrt((a ** 2).mean()), 1e-300))
    return out
