"""Seeded synthetic inputs for the pipeline-stage workloads.

This module only *generates numbers and shapes*: named stage configurations,
the flat parameter layout (names, shapes, initialisation recipe), Gaussian
tensors from a counter-based generator, ragged context lengths, shuffled page
tables, and bf16 round-trips of host arrays.  It contains none of the stage's
arithmetic, imports neither the CPU oracle nor the HIP library, and is the one
piece both sides of a parity test share.

The paper's workloads are query/reference pairs of widely varying length
(Evaluation, "Experimental Setup"); the stand-ins here are fixed-length training
micro-batches plus ragged decode contexts (uniform and clipped log-normal),
Gaussian activations and N(0, 0.02) weights.

Generator: value(seed, tensor_name, i) depends only on those three, so any
slice of any tensor can be produced in any order.
    key  = mix64(seed * G + crc32(tensor_name))
    bits = mix64(key + (2 i + j) * G),  j = 0, 1        (SplitMix64 finaliser)
    u_j  = (bits >> 11 + 0.5) / 2^53
    z    = sqrt(-2 ln u_0) * cos(2 pi u_1)               (Box-Muller, float64)
"""
from __future__ import annotations

import math
import zlib
from typing import Dict, List, Tuple

import numpy as np

_G = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 20

# --------------------------------------------------------------------------
# Stage configurations (the five workloads plus scaled-down test shapes)
# --------------------------------------------------------------------------


def _cfg(block, dtype, n_layers, d_model, n_heads, head_dim, d_ff, act,
         page_size=16, norm_eps=1e-5, rope_theta=10000.0, max_pos=4352):
    assert d_model == n_heads * head_dim
    return dict(block=block, dtype=dtype, n_layers=n_layers, d_model=d_model,
                n_heads=n_heads, head_dim=head_dim, d_ff=d_ff, act=act,
                page_size=page_size, norm_eps=norm_eps, rope_theta=rope_theta,
                max_pos=max_pos)


CONFIGS: Dict[str, dict] = {
    # 1: tiny fp32 GPT-style stage
    "tiny_gpt_f32": _cfg("gpt", "f32", 2, 128, 4, 32, 512, "gelu_tanh"),
    # 2: GPT-2-small-shaped stage
    "gpt2s_bf16": _cfg("gpt", "bf16", 6, 768, 12, 64, 3072, "gelu_tanh"),
    # 3/4: LLaMA-7B-shaped quarter model
    "llama7b_bf16": _cfg("llama", "bf16", 8, 4096, 32, 128, 11008, "swiglu"),
    # 5: LLaMA-13B-shaped quarter model
    "llama13b_bf16": _cfg("llama", "bf16", 10, 5120, 40, 128, 13824, "swiglu"),
}

# workload shapes per BASELINE config index
WORKLOADS: Dict[str, dict] = {
    "cfg1": dict(stage="tiny_gpt_f32", train=(2, 64), dy_std=1.0,
                 serve=dict(kind="prefill_decode", B=4, prompt=32, steps=16)),
    "cfg2": dict(stage="gpt2s_bf16", train=(4, 1024), dy_std=1.0,
                 serve=dict(kind="decode_fixed", B=32, ctx=512)),
    "cfg3": dict(stage="llama7b_bf16", train=(2, 2048), dy_std=1e-2, serve=None),
    "cfg4": dict(stage="llama7b_bf16", train=(1, 2048), dy_std=1e-2,
                 serve=dict(kind="decode_uniform", B=64, lo=128, hi=2048,
                            prefill_chunks=(512, 512))),
    "cfg5": dict(stage="llama13b_bf16", train=(1, 4096), dy_std=1e-2,
                 serve=dict(kind="decode_lognormal", B=128, median=1024,
                            sigma=0.7, lo=64, hi=4096)),
}


def scaled(cfg: dict, **over) -> dict:
    """Copy of a stage configuration with some fields replaced."""
    c = dict(cfg)
    c.update(over)
    assert c["d_model"] == c["n_heads"] * c["head_dim"]
    return c


# --------------------------------------------------------------------------
# Flat parameter layout (boundary order).  Every linear is [out, in] row-major.
# --------------------------------------------------------------------------


def layer_param_layout(cfg: dict) -> List[Tuple[str, Tuple[int, ...], str]]:
    """(name, shape, init) for one block, in boundary order.
    init: 'ones' | 'zeros' | 'normal' (std 0.02)."""
    d, F = cfg["d_model"], cfg["d_ff"]
    if cfg["block"] == "gpt":
        return [("ln1_g", (d,), "ones"), ("ln1_b", (d,), "zeros"),
                ("W_qkv", (3 * d, d), "normal"), ("b_qkv", (3 * d,), "zeros"),
                ("W_o", (d, d), "normal"), ("b_o", (d,), "zeros"),
                ("ln2_g", (d,), "ones"), ("ln2_b", (d,), "zeros"),
                ("W_1", (F, d), "normal"), ("b_1", (F,), "zeros"),
                ("W_2", (d, F), "normal"), ("b_2", (d,), "zeros")]
    return [("g1", (d,), "ones"), ("W_qkv", (3 * d, d), "normal"),
            ("W_o", (d, d), "normal"), ("g2", (d,), "ones"),
            ("W_gu", (2 * F, d), "normal"), ("W_d", (d, F), "normal")]


def param_layout(cfg: dict) -> List[Tuple[str, int, Tuple[int, ...], str]]:
    """(qualified name, element offset, shape, init) over the whole stage."""
    out, off = [], 0
    for l in range(cfg["n_layers"]):
        for name, shape, init in layer_param_layout(cfg):
            out.append((f"L{l}.{name}", off, shape, init))
            off += int(np.prod(shape))
    return out


def param_count(cfg: dict) -> int:
    name, off, shape, _ = param_layout(cfg)[-1]
    return off + int(np.prod(shape))


# --------------------------------------------------------------------------
# Counter-based Gaussian generator
# --------------------------------------------------------------------------


def _mix64_inplace(z: np.ndarray, tmp: np.ndarray) -> None:
    np.right_shift(z, np.uint64(30), out=tmp); np.bitwise_xor(z, tmp, out=z)
    np.multiply(z, _M1, out=z)
    np.right_shift(z, np.uint64(27), out=tmp); np.bitwise_xor(z, tmp, out=z)
    np.multiply(z, _M2, out=z)
    np.right_shift(z, np.uint64(31), out=tmp); np.bitwise_xor(z, tmp, out=z)


def _mix64_scalar(z: int) -> int:
    m = (1 << 64) - 1
    z &= m
    z = ((z ^ (z >> 30)) * int(_M1)) & m
    z = ((z ^ (z >> 27)) * int(_M2)) & m
    return z ^ (z >> 31)


def tensor_key(seed: int, name: str) -> int:
    return _mix64_scalar(seed * int(_G) + zlib.crc32(name.encode()))


def normal(seed: int, name: str, shape, std: float = 1.0, start: int = 0,
           dtype=np.float32) -> np.ndarray:
    """N(0, std^2) tensor `name`; elements [start, start+prod(shape)) of its stream."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=dtype)
    key = np.uint64(tensor_key(seed, name))
    c = min(n, _CHUNK)
    idx = np.empty(c, np.uint64); z = np.empty(c, np.uint64); tmp = np.empty(c, np.uint64)
    u0 = np.empty(c, np.float64); u1 = np.empty(c, np.float64)
    with np.errstate(over="ignore"):
        for lo in range(0, n, _CHUNK):
            m = min(_CHUNK, n - lo)
            i_, z_, t_, a_, b_ = idx[:m], z[:m], tmp[:m], u0[:m], u1[:m]
            i_[:] = np.arange(start + lo, start + lo + m, dtype=np.uint64)
            np.multiply(i_, np.uint64(2), out=i_)
            for j, u in ((0, a_), (1, b_)):
                np.add(i_, np.uint64(j), out=z_)
                np.multiply(z_, _G, out=z_)
                np.add(z_, key, out=z_)
                _mix64_inplace(z_, t_)
                np.right_shift(z_, np.uint64(11), out=z_)
                u[:] = z_
                np.add(u, 0.5, out=u)
                np.multiply(u, 1.0 / 9007199254740992.0, out=u)
            np.log(a_, out=a_); np.multiply(a_, -2.0, out=a_); np.sqrt(a_, out=a_)
            np.multiply(b_, 2.0 * math.pi, out=b_); np.cos(b_, out=b_)
            np.multiply(a_, b_, out=a_)
            if std != 1.0:
                np.multiply(a_, std, out=a_)
            out[lo:lo + m] = a_
    return out.reshape(shape)


def uniform_ints(seed: int, name: str, n: int, lo: int, hi: int) -> np.ndarray:
    """n integers uniform on [lo, hi] inclusive."""
    key = np.uint64(tensor_key(seed, name))
    with np.errstate(over="ignore"):
        z = np.arange(n, dtype=np.uint64) * _G + key
        _mix64_inplace(z, np.empty_like(z))
    u = (z >> np.uint64(11)).astype(np.float64) / 9007199254740992.0
    return (lo + np.floor(u * (hi - lo + 1))).astype(np.int64).clip(lo, hi)


def permutation(seed: int, name: str, n: int) -> np.ndarray:
    """Seeded shuffle of range(n): Fisher-Yates driven by the counter stream."""
    key = np.uint64(tensor_key(seed, name))
    with np.errstate(over="ignore"):
        z = np.arange(n, dtype=np.uint64) * _G + key
        _mix64_inplace(z, np.empty_like(z))
    r = (z >> np.uint64(11)).astype(np.float64) / 9007199254740992.0
    p = np.arange(n, dtype=np.int64)
    for i in range(n - 1, 0, -1):
        j = int(r[i] * (i + 1))
        p[i], p[j] = p[j], p[i]
    return p


# --------------------------------------------------------------------------
# bf16 round trip on the host (round-to-nearest-even), for "rounded once" inputs
# --------------------------------------------------------------------------


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 bf16 bit patterns, round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rnd) >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array whose values are exactly bf16-representable."""
    return from_bf16_bits(to_bf16_bits(x)).reshape(np.shape(x))


def quantize(x: np.ndarray, dtype: str) -> np.ndarray:
    """Values as the stage will see them: unchanged for f32, bf16-rounded for bf16."""
    return np.asarray(x, np.float32) if dtype == "f32" else round_bf16(x)


# --------------------------------------------------------------------------
# Whole-stage tensors
# --------------------------------------------------------------------------


def make_params(cfg: dict, seed: int = 0, w_std: float = 0.02,
                perturb_norm: float = 0.0) -> np.ndarray:
    """Flat float32 parameter vector in boundary order, already quantised to
    the stage dtype.  perturb_norm > 0 adds N(0, perturb_norm^2) to gains and
    biases so that tests exercise them (the configs' own recipe has gains 1,
    biases 0)."""
    flat = np.empty(param_count(cfg), np.float32)
    for name, off, shape, init in param_layout(cfg):
        n = int(np.prod(shape))
        if init == "normal":
            v = normal(seed, name, (n,), w_std)
        else:
            v = np.full(n, 1.0 if init == "ones" else 0.0, np.float32)
            if perturb_norm:
                v = v + normal(seed, name, (n,), perturb_norm)
        flat[off:off + n] = v
    return quantize(flat, cfg["dtype"])


def make_activations(cfg: dict, name: str, shape, std: float = 1.0, seed: int = 0):
    return quantize(normal(seed, name, shape, std), cfg["dtype"])


def context_lengths(serve: dict, seed: int = 0) -> np.ndarray:
    """Tokens already cached per request (the step adds one more)."""
    B = serve["B"]
    k = serve["kind"]
    if k == "decode_fixed":
        return np.full(B, serve["ctx"], np.int64)
    if k == "decode_uniform":
        return uniform_ints(seed, "ctx_len", B, serve["lo"], serve["hi"])
    if k == "decode_lognormal":
        z = normal(seed, "ctx_len", (B,), 1.0, dtype=np.float64)
        c = np.rint(np.exp(math.log(serve["median"]) + serve["sigma"] * z))
        return np.clip(c, serve["lo"], serve["hi"]).astype(np.int64)
    raise ValueError(k)


def page_tables(ctx_len: np.ndarray, new_tokens: np.ndarray, page_size: int,
                seed: int = 0, spare: float = 0.05):
    """Block table [B, max_pages] (int32, -1 = unused) over a pool whose
    physical page ids are a seeded shuffle; returns (table, n_pages)."""
    need = [int(-(-(int(c) + int(n)) // page_size)) for c, n in zip(ctx_len, new_tokens)]
    used = sum(need)
    n_pages = used + max(1, int(math.ceil(spare * used)))
    perm = permutation(seed, "page_perm", n_pages)
    table = np.full((len(need), max(need)), -1, np.int32)
    p = 0
    for b, k in enumerate(need):
        table[b, :k] = perm[p:p + k]
        p += k
    return table, n_pages


# --------------------------------------------------------------------------
# Device-side generation for the full-size workloads (billions of elements):
# torch's counter-based Philox generator seeded from (seed, tensor name).
# Values differ from normal() above but are just as reproducible; callers that
# need them on the host copy them back.
# --------------------------------------------------------------------------


def normal_torch(seed: int, name: str, shape, std: float = 1.0, device="cuda", dtype=None):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(tensor_key(seed, name) & 0x7FFFFFFFFFFFFFFF)
    x = torch.empty(tuple(shape), dtype=torch.float32, device=device)
    x.normal_(0.0, std, generator=g)
    return x if dtype is None else x.to(dtype)


def make_params_torch(cfg: dict, seed: int = 0, w_std: float = 0.02, device="cuda"):
    """Flat parameter vector on `device` in the stage's parameter dtype (the
    configs' recipe: weights N(0, w_std), gains 1, biases 0)."""
    import torch
    dt = torch.float32 if cfg["dtype"] == "f32" else torch.bfloat16
    flat = torch.empty(param_count(cfg), dtype=dt, device=device)
    for name, off, shape, init in param_layout(cfg):
        n = int(np.prod(shape))
        if init == "normal":
            flat[off:off + n] = normal_torch(seed, name, (n,), w_std, device).to(dt)
        else:
            flat[off:off + n] = 1.0 if init == "ones" else 0.0
    return flat
