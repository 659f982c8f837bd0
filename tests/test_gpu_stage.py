"""GPU parity of the stage entry points against the CPU oracle (through the C ABI).

Bar: max-abs error relative to the oracle tensor's RMS <= 1e-4 (fp32 stage) or
2e-2 (bf16 parameters, 16-bit operands, fp32 accumulation), per output tensor.
The oracle runs in float64 on the same seeded inputs, which for bf16 stages are
rounded to bf16 once on the host.
"""
import numpy as np
import pytest
import torch

from oracle import stage_oracle as O
from paper_2507_21276_amd import binding as Bd
from paper_2507_21276_amd import synth_inputs as S
import storage_rounding_model as M
from parity_util import (TOL, assert_close, dev, gather_rows_from_pool, host, param_slices,
                         pool_from_oracle_cache, rel_err)

pytestmark = pytest.mark.gpu

TD = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


def make_stage(cfg, mma=None, io=None, perturb=0.1, seed=0):
    st = Bd.Stage(cfg, io_dtype=io, mma_dtype=mma)
    flat = S.make_params(cfg, seed=seed, perturb_norm=perturb)
    assert st.ls_param_count() == flat.size
    pd = dev(flat, st.param_torch)
    st.ls_bind_params(pd)
    return st, flat, pd


def run_train(st, cfg, X, dY, B, L, accumulate_twice=False):
    T, d = B * L, cfg["d_model"]
    ws = st.new_workspace(T)
    saved = st.new_saved(B, L)
    Xd, dYd = dev(X, st.io_torch), dev(dY, st.io_torch)
    Y = torch.empty(B, L, d, dtype=st.io_torch, device="cuda")
    dX = torch.empty_like(Y)
    dP = torch.full((st.ls_param_count(),), 7.0, dtype=torch.float32, device="cuda")  # must be overwritten
    st.stage_train_fwd(Xd, B, L, Y, saved, ws)
    st.stage_train_bwd(dYd, B, L, saved, dX, dP, 0, ws)
    if accumulate_twice:
        st.stage_train_bwd(dYd, B, L, saved, dX, dP, 1, ws)
    torch.cuda.synchronize()
    return host(Y), host(dX), host(dP)


def check_train(cfg, B, L, mma, dy_std=1.0, io=None, tol=None, perturb=0.1):
    """tol: one bar for every tensor, or "storage model": per tensor, the larger of the 2e-2 bar and twice what
    bf16 storage alone costs that tensor (tests/storage_rounding_model.py)."""
    st, flat, _ = make_stage(cfg, mma=mma, io=io, perturb=perturb)
    d = cfg["d_model"]
    X = S.make_activations(cfg, "X", (B, L, d))
    dY = S.make_activations(cfg, "dY", (B, L, d), std=dy_std)
    f64 = flat.astype(np.float64)
    Yr, saved = O.stage_train_fwd(cfg, f64, X.astype(np.float64))
    dXr, dPr = O.stage_train_bwd(cfg, f64, saved, dY.astype(np.float64))
    if tol == "storage model":
        model = M.errors(cfg, (Yr, dXr, dPr), M.train(cfg, f64, X.astype(np.float64), dY.astype(np.float64),
                                                      set(M.NAMES), M.round_bf16))
        bar = lambda name: max(TOL["bf16"], 2.0 * model[name])
    else:
        bar = lambda name: tol or TOL[cfg["dtype"]]
    Y, dX, dP = run_train(st, cfg, X, dY, B, L)
    errs = {"Y": assert_close(Y, Yr, bar("Y"), "Y"), "dX": assert_close(dX, dXr, bar("dX"), "dX")}
    for name, off, n in param_slices(cfg):
        errs[name] = assert_close(dP[off:off + n], dPr[off:off + n], bar(name), "grad " + name)
    st.close()
    return errs


def test_cfg1_tiny_gpt_fp32_train_forward_backward():
    wl = S.WORKLOADS["cfg1"]
    cfg = S.CONFIGS[wl["stage"]]
    B, L = wl["train"]
    # the workload's own recipe: gains 1, biases 0
    errs = check_train(cfg, B, L, None, dy_std=wl["dy_std"], perturb=0.0)
    print("cfg1 train errors", {k: f"{v:.1e}" for k, v in list(errs.items())[:4]})
    # and with perturbed gains / biases so that those paths carry signal
    check_train(cfg, B, L, None, perturb=0.1)


def test_cfg1_tiny_gpt_fp32_prefill_then_16_decode_steps():
    wl = S.WORKLOADS["cfg1"]
    cfg = S.CONFIGS[wl["stage"]]
    sv = wl["serve"]
    Bq, N, steps, d, P = sv["B"], sv["prompt"], sv["steps"], cfg["d_model"], cfg["page_size"]
    st, flat, _ = make_stage(cfg, perturb=0.0)
    f64 = flat.astype(np.float64)
    ctx0 = np.zeros(Bq, np.int64)
    table, n_pages = S.page_tables(ctx0, np.full(Bq, N + steps), P)
    kv = Bd.KV(st, n_pages, table, ctx0)
    ws = st.new_workspace(Bq * N)
    Xp = S.make_activations(cfg, "Xprompt", (Bq, N, d))
    cache = O.new_cache(cfg, Bq)
    ys = O.stage_prefill(cfg, f64, [Xp[b].astype(np.float64) for b in range(Bq)], cache)
    Y = torch.empty(Bq * N, d, dtype=st.io_torch, device="cuda")
    st.stage_prefill(dev(Xp.reshape(Bq * N, d), st.io_torch), [N] * Bq, kv, Y, ws)
    assert_close(host(Y), np.concatenate(ys), TOL["f32"], "prefill Y")
    ctx = ctx0 + N
    for t in range(steps):
        kv.set_ctx(ctx)
        Xt = S.make_activations(cfg, f"Xdec{t}", (Bq, d))
        yr = O.stage_decode(cfg, f64, Xt.astype(np.float64), cache)
        Yt = torch.empty(Bq, d, dtype=st.io_torch, device="cuda")
        st.stage_decode(dev(Xt, st.io_torch), Bq, kv, Yt, ws)
        assert_close(host(Yt), yr, TOL["f32"], f"decode step {t}")
        ctx = ctx + 1
    # every cached K/V row agrees with the oracle's contiguous cache
    kp, vp = host(kv.k_pool), host(kv.v_pool)
    for b in range(Bq):
        Kg = gather_rows_from_pool(kp, table, b, 0, N + steps)
        Vg = gather_rows_from_pool(vp, table, b, 0, N + steps)
        for l in range(cfg["n_layers"]):
            assert_close(Kg[l], cache[l][b][0], TOL["f32"], "cached K")
            assert_close(Vg[l], cache[l][b][1], TOL["f32"], "cached V")
    st.close()


SMALL_GPT = S.scaled(S.CONFIGS["gpt2s_bf16"], n_layers=2, d_model=256, n_heads=4, d_ff=1024)
SMALL_LLAMA = S.scaled(S.CONFIGS["llama7b_bf16"], n_layers=2, d_model=256, n_heads=2, d_ff=688)


@pytest.mark.parametrize("mma", ["f16", "bf16"])
@pytest.mark.parametrize("which", ["gpt", "llama"])
def test_small_bf16_stage_train(which, mma):
    cfg = SMALL_GPT if which == "gpt" else SMALL_LLAMA
    B, L = (2, 160) if which == "gpt" else (2, 200)   # several tiles and a ragged tail
    # fp16 operands meet the 2e-2 bar.  With bf16 operands every activation and gradient the stage stores carries
    # a 2^-9 relative rounding, and that storage alone - exact arithmetic otherwise - puts 4-7e-2 into the weight
    # gradients (tests/test_storage_rounding_model.py derives it on the CPU): the bar for that mode is, per
    # tensor, the larger of 2e-2 and twice the storage model's figure.  Y and dX meet 2e-2 in both modes.
    errs = check_train(cfg, B, L, mma, dy_std=1.0 if which == "gpt" else 1e-2, io="f32",
                       tol=TOL["bf16"] if mma == "f16" else "storage model")
    if mma == "bf16":
        assert errs["Y"] <= TOL["bf16"] and errs["dX"] <= TOL["bf16"]
    print(which, mma, "worst", max(errs.items(), key=lambda kv: kv[1]))


@pytest.mark.parametrize("which", ["gpt", "llama"])
def test_small_bf16_stage_train_with_bf16_io(which):
    # Y and dX leave the stage in bf16: the final rounding alone can reach
    # 2^-8 of the largest element, so this variant is held to 2e-2 + that bound.
    cfg = SMALL_GPT if which == "gpt" else SMALL_LLAMA
    st, flat, _ = make_stage(cfg, mma="f16", io="bf16")
    B, L, d = 2, 96, cfg["d_model"]
    X = S.make_activations(cfg, "X", (B, L, d))
    dY = S.make_activations(cfg, "dY", (B, L, d))
    Yr, saved = O.stage_train_fwd(cfg, flat.astype(np.float64), X.astype(np.float64))
    dXr, _ = O.stage_train_bwd(cfg, flat.astype(np.float64), saved, dY.astype(np.float64))
    Y, dX, _ = run_train(st, cfg, X, dY, B, L)
    for got, ref, nm in ((Y, Yr, "Y"), (dX, dXr, "dX")):
        rms = np.sqrt((ref ** 2).mean())
        assert_close(got, ref, 2e-2 + 2.0 ** -8 * np.abs(ref).max() / rms, nm)
        assert_close(got, S.round_bf16(ref.astype(np.float32)), 2e-2, nm + " vs rounded oracle")
    st.close()


def test_deep_llama_stage_meets_tolerance_with_fp16_operands():
    # eight blocks, the depth of the LLaMA-7B-shaped stage, at reduced width
    cfg = S.scaled(S.CONFIGS["llama7b_bf16"], n_layers=8, d_model=512, n_heads=4, d_ff=1376)
    errs = check_train(cfg, 1, 192, "f16", dy_std=1e-2, io="f32", perturb=0.0)
    print("deep llama f16 worst", max(errs.items(), key=lambda kv: kv[1]))


def test_accumulate_adds_microbatch_gradients():
    cfg = SMALL_LLAMA
    st, flat, _ = make_stage(cfg, mma="f16", io="f32")
    B, L, d = 1, 64, cfg["d_model"]
    X = S.make_activations(cfg, "X", (B, L, d))
    dY = S.make_activations(cfg, "dY", (B, L, d))
    _, _, g1 = run_train(st, cfg, X, dY, B, L)
    _, _, g2 = run_train(st, cfg, X, dY, B, L, accumulate_twice=True)
    assert_close(g2, 2.0 * g1, 1e-6, "accumulated gradient")
    st.close()


def serve_case(cfg, mma, ctx, new, seed=0, junk_kind="gauss"):
    """Direct-filled cache (seeded N(0,1) K/V per layer), then one call with
    `new[b]` new tokens per request; returns (gpu Y, oracle Y, errors on new KV rows)."""
    st, flat, _ = make_stage(cfg, mma=mma, io="f32" if cfg["dtype"] == "bf16" else None)
    f64 = flat.astype(np.float64)
    d, P, nL, h, dh = cfg["d_model"], cfg["page_size"], cfg["n_layers"], cfg["n_heads"], cfg["head_dim"]
    Bq = len(ctx)
    table, n_pages = S.page_tables(ctx, new, P, seed=seed)
    kv = Bd.KV(st, n_pages, table, ctx)
    qt = (lambda a: a.astype(np.float16).astype(np.float32)) if mma == "f16" else (lambda a: S.quantize(a, cfg["dtype"]))
    cache = O.new_cache(cfg, Bq)
    for l in range(nL):
        for b in range(Bq):
            K = qt(S.normal(seed, f"K{l}.{b}", (int(ctx[b]), h, dh)))
            V = qt(S.normal(seed, f"V{l}.{b}", (int(ctx[b]), h, dh)))
            cache[l][b] = [K.astype(np.float64), V.astype(np.float64)]
    kp, vp = pool_from_oracle_cache(cache, table, n_pages, cfg)
    # unused slots hold garbage that must not leak into any result
    junk = np.random.default_rng(1).normal(0, 50, kp.shape).astype(np.float32)
    if junk_kind == "nan":
        junk[:] = np.nan
    elif junk_kind == "inf":
        junk[:] = np.where(junk > 0, np.inf, -np.inf)
    used = np.zeros(kp.shape[:2] + (1, P, 1), bool)
    for b in range(Bq):
        for j in range(int(ctx[b])):
            used[:, table[b, j // P], 0, j % P, 0] = True
    kp = np.where(used, kp, junk); vp = np.where(used, vp, junk)
    kv.k_pool.copy_(dev(kp, kv.k_pool.dtype)); kv.v_pool.copy_(dev(vp, kv.v_pool.dtype))
    T = int(np.sum(new))
    X = S.make_activations(cfg, "Xserve", (T, d))
    chunks, t0 = [], 0
    for b in range(Bq):
        chunks.append(X[t0:t0 + new[b]].astype(np.float64)); t0 += new[b]
    ys = O.stage_prefill(cfg, f64, chunks, cache)
    ws = st.new_workspace(T)
    Y = torch.empty(T, d, dtype=st.io_torch, device="cuda")
    if all(n == 1 for n in new):
        st.stage_decode(dev(X, st.io_torch), Bq, kv, Y, ws)
    else:
        st.stage_prefill(dev(X, st.io_torch), list(new), kv, Y, ws)
    torch.cuda.synchronize()
    kph, vph = host(kv.k_pool), host(kv.v_pool)
    kv_err = 0.0
    for b in range(Bq):
        lo, hi = int(ctx[b]), int(ctx[b] + new[b])
        Kg = gather_rows_from_pool(kph, table, b, lo, hi)
        Vg = gather_rows_from_pool(vph, table, b, lo, hi)
        for l in range(nL):
            kv_err = max(kv_err, rel_err(Kg[l], cache[l][b][0][lo:hi]), rel_err(Vg[l], cache[l][b][1][lo:hi]))
    st.close()
    return host(Y), np.concatenate(ys), kv_err


@pytest.mark.parametrize("which,mma", [("gpt", "f16"), ("llama", "f16"), ("llama", "bf16")])
def test_ragged_decode_over_shuffled_pages(which, mma):
    cfg = SMALL_GPT if which == "gpt" else SMALL_LLAMA
    ctx = np.array([0, 1, 15, 16, 17, 100, 333, 257, 64, 31])
    Y, Yr, kv_err = serve_case(cfg, mma, ctx, np.ones_like(ctx))
    assert_close(Y, Yr, TOL["bf16"], "decode Y")
    assert kv_err <= TOL["bf16"]


@pytest.mark.parametrize("junk", ["nan", "inf"])
def test_unwritten_page_slots_may_hold_nan_or_infinity(junk):
    """A caller may hand over pools straight from the allocator: the slots of a last page beyond the context,
    and the spare pages, hold NaN or infinities here.  Decode steps and prompt chunks give the oracle's result."""
    ctx = np.array([0, 1, 15, 16, 17, 100, 333, 257, 64, 31])
    Y, Yr, kv_err = serve_case(SMALL_LLAMA, "f16", ctx, np.ones_like(ctx), junk_kind=junk)
    assert np.isfinite(Y).all()
    assert_close(Y, Yr, TOL["bf16"], "decode Y")
    assert kv_err <= TOL["bf16"]
    Y, Yr, kv_err = serve_case(SMALL_LLAMA, "f16", np.array([0, 128, 37, 5]), np.array([96, 64, 1, 130]), junk_kind=junk)
    assert np.isfinite(Y).all()
    assert_close(Y, Yr, TOL["bf16"], "prefill Y")
    assert kv_err <= TOL["bf16"]


@pytest.mark.parametrize("which", ["gpt", "llama"])
def test_prefill_chunks_with_past_and_mixed_lengths(which):
    cfg = SMALL_GPT if which == "gpt" else SMALL_LLAMA
    ctx = np.array([0, 128, 37, 5])
    new = np.array([96, 64, 1, 130])
    Y, Yr, kv_err = serve_case(cfg, "f16", ctx, new)
    assert_close(Y, Yr, TOL["bf16"], "prefill Y")
    assert kv_err <= TOL["bf16"]


def test_chunked_prefill_equals_single_prefill_and_train_forward():
    cfg = SMALL_LLAMA
    st, flat, _ = make_stage(cfg, mma="f16", io="f32")
    d, P, N = cfg["d_model"], cfg["page_size"], 160
    X = S.make_activations(cfg, "X", (N, d))
    Xd = dev(X, st.io_torch)
    ws = st.new_workspace(N)
    outs = []
    for chunks in ([N], [64, 96]):
        table, n_pages = S.page_tables(np.zeros(1, np.int64), np.array([N]), P)
        kv = Bd.KV(st, n_pages, table, [0])
        Y = torch.empty(N, d, dtype=st.io_torch, device="cuda")
        t0 = 0
        for c in chunks:
            kv.set_ctx([t0])
            st.stage_prefill(Xd[t0:t0 + c], [c], kv, Y[t0:t0 + c], ws)
            t0 += c
        outs.append(host(Y))
    saved = st.new_saved(1, N)
    Yt = torch.empty(1, N, d, dtype=st.io_torch, device="cuda")
    st.stage_train_fwd(Xd, 1, N, Yt, saved, ws)
    Yr, _ = O.stage_train_fwd(cfg, flat.astype(np.float64), X[None].astype(np.float64))
    for y, nm in ((outs[0], "single prefill"), (outs[1], "chunked prefill"), (host(Yt)[0], "train fwd")):
        assert_close(y, Yr[0], TOL["bf16"], nm)
    assert_close(outs[1], outs[0], 5e-3, "chunked vs single")
    st.close()


def test_host_validation_of_serving_arguments():
    cfg = SMALL_LLAMA
    st, _, _ = make_stage(cfg, mma="f16", io="f32")
    table, n_pages = S.page_tables(np.array([30]), np.array([1]), cfg["page_size"])
    kv = Bd.KV(st, n_pages, table, [30])
    ws = st.new_workspace(64)
    X = torch.zeros(64, cfg["d_model"], dtype=st.io_torch, device="cuda")
    Y = torch.zeros_like(X)
    kv.set_ctx([32])                       # 33 tokens need 3 pages, table holds 2
    with pytest.raises(Bd.LsError) as e:
        st.stage_decode(X, 1, kv, Y, ws)
    assert e.value.status == Bd.LS_EINVAL and "pages" in str(e.value)
    kv.set_ctx([0])
    with pytest.raises(Bd.LsError):
        st.stage_prefill(X, [64], kv, Y, ws)   # 64 tokens > 2 pages
    with pytest.raises(Bd.LsError):
        st.stage_prefill(X, [0], kv, Y, ws)
    unbound = Bd.Stage(cfg, io_dtype="f32", mma_dtype="f16")
    with pytest.raises(Bd.LsError) as e:
        unbound.stage_decode(X, 1, kv, Y, ws)
    assert e.value.status == Bd.LS_ESTATE
    st.close(); unbound.close()


def hybrid_case(cfg, mma, ctx, new, n_decode, seed=3):
    """As serve_case, through stage_step: the first n_decode requests decode one token, the rest
    bring a prompt chunk.  The oracle treats every request as a chunk (single-token chunks for
    the decode rows): rows of different requests never mix."""
    st, flat, _ = make_stage(cfg, mma=mma, io="f32" if cfg["dtype"] == "bf16" else None)
    f64 = flat.astype(np.float64)
    d, P, nL, h, dh = cfg["d_model"], cfg["page_size"], cfg["n_layers"], cfg["n_heads"], cfg["head_dim"]
    Bq = len(ctx)
    assert all(n == 1 for n in new[:n_decode])
    table, n_pages = S.page_tables(ctx, new, P, seed=seed)
    kv = Bd.KV(st, n_pages, table, ctx)
    qt = ((lambda a: a.astype(np.float16).astype(np.float32)) if mma == "f16" else
          (lambda a: S.quantize(a, cfg["dtype"])) if mma else (lambda a: a.astype(np.float32)))
    cache = O.new_cache(cfg, Bq)
    for l in range(nL):
        for b in range(Bq):
            K = qt(S.normal(seed, f"K{l}.{b}", (int(ctx[b]), h, dh)))
            V = qt(S.normal(seed, f"V{l}.{b}", (int(ctx[b]), h, dh)))
            cache[l][b] = [K.astype(np.float64), V.astype(np.float64)]
    kp, vp = pool_from_oracle_cache(cache, table, n_pages, cfg)
    kv.k_pool.copy_(dev(kp, kv.k_pool.dtype))
    kv.v_pool.copy_(dev(vp, kv.v_pool.dtype))
    T = int(np.sum(new))
    X = S.make_activations(cfg, "Xh", (T, d))
    chunks, t0 = [], 0
    for b in range(Bq):
        chunks.append(X[t0:t0 + new[b]].astype(np.float64)); t0 += new[b]
    ys = O.stage_prefill(cfg, f64, chunks, cache)
    Y = torch.empty(T, d, dtype=st.io_torch, device="cuda")
    st.stage_step(dev(X, st.io_torch), n_decode, list(new[n_decode:]), kv, Y, st.new_workspace(T))
    torch.cuda.synchronize()
    kph, vph = host(kv.k_pool), host(kv.v_pool)
    kv_err = 0.0
    for b in range(Bq):
        lo, hi = int(ctx[b]), int(ctx[b] + new[b])
        Kg = gather_rows_from_pool(kph, table, b, lo, hi)
        Vg = gather_rows_from_pool(vph, table, b, lo, hi)
        for l in range(nL):
            kv_err = max(kv_err, rel_err(Kg[l], cache[l][b][0][lo:hi]), rel_err(Vg[l], cache[l][b][1][lo:hi]))
    st.close()
    return host(Y), np.concatenate(ys), kv_err


@pytest.mark.parametrize("which,mma", [("llama", "f16"), ("gpt", "f16"), ("llama", "bf16"), ("tiny", None)])
def test_hybrid_batch_of_decode_rows_and_prompt_chunks(which, mma):
    cfg = {"llama": SMALL_LLAMA, "gpt": SMALL_GPT, "tiny": S.CONFIGS["tiny_gpt_f32"]}[which]
    ctx = np.array([5, 0, 100, 31, 257, 16, 0, 40, 130])
    new = np.array([1, 1, 1, 1, 1, 1, 70, 300, 33])
    Y, Yr, kv_err = hybrid_case(cfg, mma, ctx, new, n_decode=6)
    tol = TOL["bf16"] if mma else TOL["f32"]
    assert_close(Y, Yr, tol, "hybrid Y")
    # K / V rows stored in bf16 carry half an ulp of their largest element (about 4 RMS): 2^-9 * 4 on top of the bar
    assert kv_err <= tol + (2.0 ** -7 if mma == "bf16" else 0.0)
    # degenerate mixes: decode rows only, prompt chunks only
    Y, Yr, _ = hybrid_case(cfg, mma, ctx[:6], new[:6], n_decode=6)
    assert_close(Y, Yr, tol, "hybrid, decode rows only")
    Y, Yr, _ = hybrid_case(cfg, mma, ctx[6:], new[6:], n_decode=0)
    assert_close(Y, Yr, tol, "hybrid, prompt chunks only")


def test_hybrid_batch_rejects_bad_arguments():
    cfg = SMALL_LLAMA
    st, _, _ = make_stage(cfg, mma="f16", io="f32")
    table, n_pages = S.page_tables(np.array([0, 0]), np.array([1, 8]), cfg["page_size"])
    kv = Bd.KV(st, n_pages, table, [0, 0])
    X = torch.zeros(9, cfg["d_model"], device="cuda")
    ws = st.new_workspace(16)
    with pytest.raises(Bd.LsError):
        st.stage_step(X, 0, [], kv, X, ws)                 # empty batch
    with pytest.raises(Bd.LsError):
        st.stage_step(X, 1, [0], kv, X, ws)                # empty chunk
    with pytest.raises(Bd.LsError):
        st.stage_step(X, 1, [8] * 33, kv, X, ws)           # too many chunks
    st.close()
