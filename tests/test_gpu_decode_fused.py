"""Decode-batch projections that leave split-K partial products, and the kernels that sum them
and apply the step that follows the projection (rotary embedding + K/V page write, residual +
normalisation, activation): each against the float64 oracle, then whole decode steps of small
stages whose widths take this path."""
import numpy as np
import pytest
import torch

from oracle import stage_oracle as O
from paper_2507_21276_amd import binding as Bd
from paper_2507_21276_amd import synth_inputs as S
from parity_util import (TOL, assert_close, dev, gather_rows_from_pool, host, out_rounding_bound,
                         pool_from_oracle_cache, rel_err)

pytestmark = pytest.mark.gpu

DT = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


def q(a, name):
    return dev(a, DT[name]).float().cpu().numpy().astype(np.float64)


def rope_table(max_pos, dh, theta=1e4):
    i = np.arange(dh // 2, dtype=np.float64)
    ang = np.arange(max_pos, dtype=np.float64)[:, None] * theta ** (-2.0 * i / dh)[None, :]
    return np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)


def partials_of(name, M, N, K, seed, floats=None):
    x = S.normal_torch(seed, "x", (M, K), 1.0, dtype=DT[name])
    w = S.normal_torch(seed, "w", (N, K), K ** -0.5, dtype=DT[name])
    part = torch.full((floats or 16 * M * N,), float("nan"), dtype=torch.float32, device="cuda")
    splits = Bd.lsk_gemm_partials(x, w, part)
    return x, w, part, splits


@pytest.mark.parametrize("name", ["f16", "bf16"])
@pytest.mark.parametrize("M,N,K", [(64, 4096, 4096), (64, 12288, 4096), (33, 264, 1024), (1, 128, 512),
                                   (64, 4096, 11008), (7, 1048, 704), (128, 5120, 5120), (100, 27648, 5120),
                                   (65, 264, 1024)])
def test_partials_sum_to_the_product(name, M, N, K):
    x, w, part, splits = partials_of(name, M, N, K, 41)
    assert 1 <= splits <= 16
    got = host(part[:splits * M * N].view(splits, M, N)).sum(0)
    ref = host(x) @ host(w).T
    assert_close(got, ref, 1e-5, "sum of partials")
    # a buffer that holds one result only: one split
    _, _, part1, s1 = partials_of(name, M, N, K, 41, floats=M * N)
    assert s1 == 1
    assert_close(host(part1.view(M, N)), ref, 1e-5, "single split")
    with pytest.raises(Bd.LsError):
        partials_of(name, 129, N, K, 41)
    with pytest.raises(Bd.LsError):
        partials_of(name, M, N, K, 41, floats=M * N - 4)


@pytest.mark.parametrize("kind", [0, 1, -1])
@pytest.mark.parametrize("name", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("T,d,splits", [(64, 4096, 10), (5, 768, 1), (33, 1600, 3)])
def test_finish_residual_and_norm(kind, name, T, d, splits):
    part = S.normal(42, "part", (splits, T, d))
    bias = q(S.normal(42, "bias", (d,), 0.1), "bf16")
    resid = S.normal(42, "resid", (T, d))
    g = q(1.0 + S.normal(42, "g", (d,), 0.1), "bf16")
    b = q(S.normal(42, "b", (d,), 0.1), "bf16")
    x_ref = part.astype(np.float32).astype(np.float64).sum(0) + bias + resid.astype(np.float32)
    x_out = torch.empty(T, d, dtype=torch.float32, device="cuda")
    h = torch.empty(T, d, dtype=DT[name], device="cuda")
    Bd.lsk_finish_resid_norm(dev(part, torch.float32), splits, T, d, x_out, bias=dev(bias, torch.bfloat16),
                             resid=dev(resid, torch.float32), kind=kind, gamma=dev(g, torch.bfloat16),
                             beta=dev(b, torch.bfloat16) if kind == 0 else None, h=h)
    assert_close(host(x_out), x_ref, 1e-6, "x_out")
    if kind >= 0:
        ref = O.layer_norm(x_ref, g, b, 1e-5)[0] if kind == 0 else O.rms_norm(x_ref, g, 1e-5)[0]
        tol = 1e-5 if name == "f32" else 1e-4 + out_rounding_bound(ref, name)
        assert_close(host(h), ref, tol, "normalised output")
    # no bias, no residual, in place over the residual buffer
    x2 = dev(resid, torch.float32)
    Bd.lsk_finish_resid_norm(dev(part, torch.float32), splits, T, d, x2, resid=x2, kind=-1)
    assert_close(host(x2), x_ref - bias, 1e-6, "in place")


@pytest.mark.parametrize("name", ["f16", "bf16"])
@pytest.mark.parametrize("act,T,F,splits", [("swiglu", 64, 11008, 4), ("swiglu", 3, 704, 1), ("gelu_tanh", 40, 1024, 7),
                                            ("gelu_erf", 9, 3072, 2)])
def test_finish_activation(name, act, T, F, splits):
    cols = 2 * F if act == "swiglu" else F
    part = S.normal(43, "part", (splits, T, cols), 0.7)
    bias = q(S.normal(43, "bias", (cols,), 0.1), "bf16")
    z = part.astype(np.float32).astype(np.float64).sum(0) + bias
    ref = O.silu(z[:, :F]) * z[:, F:] if act == "swiglu" else O.gelu(z, act)
    out = torch.empty(T, F, dtype=DT[name], device="cuda")
    Bd.lsk_finish_act(dev(part, torch.float32), splits, T, F, Bd.ACT_CODE[act], out, bias=dev(bias, torch.bfloat16))
    assert_close(host(out), ref, 1e-4 + out_rounding_bound(ref, name), "activation")


@pytest.mark.parametrize("name,h,dh,P,rope,with_bias", [("f16", 2, 128, 16, True, False), ("bf16", 3, 64, 8, True, False),
                                                      ("f16", 4, 32, 16, False, True)])
def test_finish_qkv_rotary_and_page_write(name, h, dh, P, rope, with_bias):
    d = h * dh
    ctx = np.array([0, 5, 16, 100, 333, 47])
    new = np.array([1, 1, 3, 1, 20, 4])
    T, splits = int(new.sum()), 5
    table, n_pages = S.page_tables(ctx, new, P, seed=3)
    pos = np.concatenate([ctx[b] + np.arange(new[b]) for b in range(len(ctx))]).astype(np.int32)
    req = np.concatenate([np.full(new[b], b) for b in range(len(ctx))]).astype(np.int32)
    part = S.normal(44, "part", (splits, T, 3 * d), 0.5)
    bias = q(S.normal(44, "bias", (3 * d,), 0.1), "bf16")
    z = part.astype(np.float32).astype(np.float64).sum(0) + (bias if with_bias else 0.0)
    ref = z.copy()
    if rope:
        for part_i in (0, 1):
            blk = z[:, part_i * d:(part_i + 1) * d].reshape(T, h, dh)
            ref[:, part_i * d:(part_i + 1) * d] = O.rope(blk, pos, 1e4, 1.0).reshape(T, d)
    rng = np.random.default_rng(1)
    kp0 = rng.normal(0, 1, (n_pages, h, P, dh))
    kd, vd = dev(kp0, DT[name]), dev(kp0 * 2, DT[name])
    k_before = host(kd)
    qkv = torch.empty(T, 3 * d, dtype=DT[name], device="cuda")
    Bd.lsk_finish_qkv(dev(part, torch.float32), splits, h, dh, torch.as_tensor(pos, device="cuda"),
                      torch.as_tensor(req, device="cuda"), dev(rope_table(512, dh), torch.float32) if rope else None,
                      qkv, kd, vd, torch.as_tensor(table, dtype=torch.int32, device="cuda"), P,
                      bias=dev(bias, torch.bfloat16) if with_bias else None)
    got = host(qkv)
    assert_close(got, ref, 1e-5 + out_rounding_bound(ref, name), "q | k | v")
    # the K and V rows in the pages are the 16-bit values of the qkv buffer, bit for bit; nothing else moved
    kh, vh = host(kd), host(vd)
    touched = np.zeros(kh.shape[:1] + kh.shape[2:3], bool)
    for t in range(T):
        pg, slot = table[req[t], pos[t] // P], pos[t] % P
        assert np.array_equal(kh[pg, :, slot], got[t, d:2 * d].reshape(h, dh))
        assert np.array_equal(vh[pg, :, slot], got[t, 2 * d:].reshape(h, dh))
        touched[pg, slot] = True
    assert np.array_equal(kh[~touched[:, None, :].repeat(h, 1)], k_before[~touched[:, None, :].repeat(h, 1)])


FUSED_LLAMA = S.scaled(S.CONFIGS["llama7b_bf16"], n_layers=3, d_model=256, n_heads=2, d_ff=704)
FUSED_GPT = S.scaled(S.CONFIGS["gpt2s_bf16"], n_layers=3, d_model=256, n_heads=4, d_ff=1024)


@pytest.mark.parametrize("which,mma", [("llama", "f16"), ("gpt", "f16"), ("llama", "bf16")])
def test_decode_steps_of_a_stage_whose_widths_take_the_fused_path(which, mma):
    """Widths that are multiples of 64: serving calls of at most 64 rows run the partial-product
    projections and the fused finish kernels; three blocks, so the normalisation handed from one
    block to the next is covered.  A ragged batch decodes three steps, then a short prompt chunk
    and more decode rows share one hybrid call."""
    cfg = FUSED_LLAMA if which == "llama" else FUSED_GPT
    st = Bd.Stage(cfg, io_dtype="f32", mma_dtype=mma)
    flat = S.make_params(cfg, seed=0, perturb_norm=0.1)
    st.ls_bind_params(dev(flat, st.param_torch))
    f64 = flat.astype(np.float64)
    d, P, nL, h, dh = cfg["d_model"], cfg["page_size"], cfg["n_layers"], cfg["n_heads"], cfg["head_dim"]
    ctx = np.array([5, 0, 100, 31, 257, 16, 40])
    Bq, steps = len(ctx), 3
    table, n_pages = S.page_tables(ctx, np.full(Bq, steps + 24), P, seed=4)
    kv = Bd.KV(st, n_pages, table, ctx)
    qt = ((lambda a: a.astype(np.float16).astype(np.float32)) if mma == "f16" else (lambda a: S.quantize(a, cfg["dtype"])))
    cache = O.new_cache(cfg, Bq)
    for l in range(nL):
        for b in range(Bq):
            cache[l][b] = [qt(S.normal(5, f"K{l}.{b}", (int(ctx[b]), h, dh))).astype(np.float64),
                           qt(S.normal(5, f"V{l}.{b}", (int(ctx[b]), h, dh))).astype(np.float64)]
    kp, vp = pool_from_oracle_cache(cache, table, n_pages, cfg)
    kv.k_pool.copy_(dev(kp, kv.k_pool.dtype))
    kv.v_pool.copy_(dev(vp, kv.v_pool.dtype))
    tol = TOL["bf16"] if mma == "f16" else 1e-1
    ws = st.new_workspace(64)
    cur = ctx.copy()
    for step in range(steps):
        X = S.make_activations(cfg, f"Xd{step}", (Bq, d))
        ref = O.stage_decode(cfg, f64, X.astype(np.float64), cache)
        Y = torch.empty(Bq, d, dtype=st.io_torch, device="cuda")
        kv.set_ctx(cur)
        st.stage_decode(dev(X, st.io_torch), Bq, kv, Y, ws)
        assert_close(host(Y), ref, tol, f"decode step {step}")
        cur = cur + 1
    # hybrid call: every request but the last decodes once more, the last one brings a 20-token chunk
    new = np.ones(Bq, dtype=np.int64)
    new[-1] = 20
    T = int(new.sum())
    X = S.make_activations(cfg, "Xh", (T, d))
    chunks, t0 = [], 0
    for b in range(Bq):
        chunks.append(X[t0:t0 + new[b]].astype(np.float64)); t0 += new[b]
    ys = O.stage_prefill(cfg, f64, chunks, cache)
    Y = torch.empty(T, d, dtype=st.io_torch, device="cuda")
    kv.set_ctx(cur)
    st.stage_step(dev(X, st.io_torch), Bq - 1, [20], kv, Y, ws)
    assert_close(host(Y), np.concatenate(ys), tol, "hybrid call of 26 rows")
    torch.cuda.synchronize()
    kph = host(kv.k_pool)
    for b in range(Bq):
        lo, hi = int(ctx[b]), int(cur[b] + new[b])
        Kg = gather_rows_from_pool(kph, table, b, lo, hi)
        for l in range(nL):
            assert rel_err(Kg[l], cache[l][b][0][lo:hi]) <= tol
    st.close()
