#!/usr/bin/env python3
"""Benchmark of the pipeline-stage hot path on one MI355X.

One *step* is one pass of the whole hot path on the LLaMA-7B-shaped 8-block
stage (bf16 parameters, 16-bit matrix-core operands, fp32 accumulation):
  1. a training micro-batch of 2 x 2048 tokens, forward + backward
     (stage_train_fwd + stage_train_bwd),
  2. one ragged decode step for 64 requests, contexts uniform in [128, 2048],
     16-token pages in shuffled order (stage_decode),
  3. two 512-token prefill chunks of one 1024-token prompt (stage_prefill x 2).
All inputs are seeded, synthetic and resident in HBM before the timed region.
`value` is tokens processed per second over the whole step; the per-leg rates,
the GEMM roofline (from HIP events around the stage's own GEMM launches, recorded by the
library in a pass of its own), the decode roofline, the same legs with the other operand
format, the two-stream interference probe and the CPU oracle baseline are reported beside
it on the same JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--mma f16|bf16]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_TFLOPS = 2500.0   # dense bf16 / fp16 MFMA, MI355X
PEAK_HBM_GBS = 8000.0       # HBM3E


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_events(torch, fn, iters, warm=1):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def cpu_baseline(cfg, S):
    """The oracle, as it stands, on a bounded sample of the training workload."""
    from oracle import stage_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    nl, L = 2, 2048
    c = S.scaled(cfg, n_layers=nl)
    flat = S.make_params(c).astype(np.float64)
    X = S.make_activations(c, "X", (1, L, c["d_model"])).astype(np.float64)
    dY = S.make_activations(c, "dY", (1, L, c["d_model"]), std=1e-2).astype(np.float64)
    t0 = time.perf_counter()
    _, saved = O.stage_train_fwd(c, flat, X)
    O.stage_train_bwd(c, flat, saved, dY)
    dt = time.perf_counter() - t0
    scale = cfg["n_layers"] / nl
    return {"value": L / (dt * scale), "unit": "tok/s", "cores": int(cores), "kind": "oracle",
            "sample": f"train fwd+bwd of {nl} of {cfg['n_layers']} blocks on 1x{L} tokens in float64 numpy "
                      f"({dt:.1f} s), time scaled x{scale:g} to the full stage"}


def gemm_study():
    """C[4096, 4096] = A B^T in fp16 for K = 1024 .. 8192: microseconds per launch for `lsk_gemm` and for
    torch.matmul (the vendor library), first with all-zero operands (no data toggling, the clock stays up),
    then with N(0,1) operands.  The slope over K is the cost of a 64-wide k tile, the intercept the fixed
    cost of a launch (first loads, ramp, epilogue)."""
    import torch
    from paper_2507_21276_amd import binding as Bd

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    Bd.lib()

    def timed(fn, iters=100, warm=10):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters * 1e3

    M = N = 4096
    out = {}
    for kind in ("zeros", "normal"):
        rows = []
        for K in (1024, 2048, 4096, 8192):
            if kind == "zeros":
                A = torch.zeros(M, K, device="cuda", dtype=torch.float16)
                B = torch.zeros(N, K, device="cuda", dtype=torch.float16)
            else:
                g = torch.Generator(device="cuda").manual_seed(K)
                A = torch.randn(M, K, device="cuda", generator=g).to(torch.float16)
                B = torch.randn(N, K, device="cuda", generator=g).to(torch.float16)
            C = torch.empty(M, N, device="cuda", dtype=torch.float16)
            ours = timed(lambda: Bd.lsk_gemm(A, B, C, M=M, N=N, K=K))
            lib = timed(lambda: torch.matmul(A, B.T, out=C))
            rows.append((K, ours, lib))
            print(f"{kind:6s} K={K:5d}: lsk_gemm {ours:7.1f} us ({2 * M * N * K / ours / 1e6:5.0f} TFLOP/s)   "
                  f"torch.matmul {lib:7.1f} us ({2 * M * N * K / lib / 1e6:5.0f} TFLOP/s)", flush=True)
        (k0, a0, b0), (k1, a1, b1) = rows[2], rows[3]
        sa, sb = (a1 - a0) / (k1 - k0) * 64, (b1 - b0) / (k1 - k0) * 64
        print(f"{kind:6s} per 64-wide k tile (K 4096 -> 8192): lsk_gemm {sa:.3f} us, torch.matmul {sb:.3f} us; "
              f"fixed per launch: lsk_gemm {a0 - sa * k0 / 64:.1f} us, torch.matmul {b0 - sb * k0 / 64:.1f} us", flush=True)
        out[kind] = {"k_tile_us": [sa, sb], "fixed_us": [a0 - sa * k0 / 64, b0 - sb * k0 / 64]}
    # the gradient layouts at the four projection shapes of a LLaMA-7B block (T = 4096 tokens, N(0, 0.05) / N(0, 1)
    # operands): weight gradient dW[M, N] = dY[T, M]^T X[T, N] (both operands k-strided; fp32 result from
    # lsk_gemm, fp16 from torch.matmul) and input gradient dX[T, N] = dY[T, M] W[M, N] (W k-strided)
    T = 4096
    layouts = []
    for (Mo, No) in ((4096, 11008), (4096, 4096), (22016, 4096), (12288, 4096)):
        g = torch.Generator(device="cuda").manual_seed(1)
        dY = (torch.randn(T, Mo, device="cuda", generator=g) * 0.05).to(torch.float16)
        X = torch.randn(T, No, device="cuda", generator=g).to(torch.float16)
        W = (torch.randn(Mo, No, device="cuda", generator=g) * 0.05).to(torch.float16)
        C32 = torch.zeros(Mo, No, device="cuda", dtype=torch.float32)
        C16 = torch.zeros(Mo, No, device="cuda", dtype=torch.float16)
        dX = torch.zeros(T, No, device="cuda", dtype=torch.float16)
        fl = 2.0 * Mo * No * T
        row = {"shape": [Mo, No]}
        for name, ours, lib in (
                ("dW", lambda: Bd.lsk_gemm(dY, X, C32, M=Mo, N=No, K=T, a_kmajor=False, b_kmajor=False),
                 lambda: torch.matmul(dY.T, X, out=C16)),
                ("dW+=", lambda: Bd.lsk_gemm(dY, X, C32, M=Mo, N=No, K=T, a_kmajor=False, b_kmajor=False, accumulate=True),
                 None),
                ("dX", lambda: Bd.lsk_gemm(dY, W, dX, M=T, N=No, K=Mo, a_kmajor=True, b_kmajor=False),
                 lambda: torch.matmul(dY, W, out=dX))):
            a = timed(ours, iters=50, warm=5)
            b = timed(lib, iters=50, warm=5) if lib else None
            row[name] = [a, b]
            print(f"{name:4s} {Mo:5d} x {No:5d}: lsk_gemm {a:7.1f} us ({fl / a / 1e6:5.0f} TFLOP/s)"
                  + (f"   torch.matmul {b:7.1f} us ({fl / b / 1e6:5.0f} TFLOP/s)" if b else ""), flush=True)
        layouts.append(row)
    print(json.dumps({"gemm_study": out, "gradient_layouts": layouts}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--mma", default="f16", choices=["f16", "bf16"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe", action="store_true")
    ap.add_argument("--no-cfg5", action="store_true", help="skip the config-5 decode measurement")
    ap.add_argument("--no-serve-loop", action="store_true", help="skip the continuous-batching loop measurement")
    ap.add_argument("--no-other-mode", action="store_true", help="skip the legs with the other operand format")
    ap.add_argument("--no-update", action="store_true", help="skip the model-update measurement (3 fp32 vectors of the stage's size)")
    ap.add_argument("--legs", default="train,decode,prefill",
                    help="comma list of the legs that make up a step (profiling aid; the default is the full "
                         "step; 'gemms' = the 12 GEMM launches of one block on their own; 'calib' = a 256 MiB copy kernel "
                         "used to scale the HBM byte counters)")
    ap.add_argument("--gemm-study", action="store_true",
                    help="instead of the step: time the GEMM kernel over contraction lengths with all-zero and with "
                         "N(0,1) operands (the chip clocks down on real data) beside torch.matmul, print a table and exit")
    args = ap.parse_args()
    if args.gemm_study:
        return gemm_study()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (one pipeline stage on one MI355X); "
                 "run with --gpus 1")

    import torch
    from paper_2507_21276_amd import binding as Bd
    from paper_2507_21276_amd import synth_inputs as S

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    Bd.lib()   # fails loudly when the HIP library has not been built
    dev = "cuda"
    cfg = S.CONFIGS["llama7b_bf16"]
    d, nL, F, h, dh, P = (cfg[k] for k in ("d_model", "n_layers", "d_ff", "n_heads", "head_dim", "page_size"))
    st = Bd.Stage(cfg, io_dtype="bf16", mma_dtype=args.mma)
    params = S.make_params_torch(cfg, seed=0, device=dev)
    st.ls_bind_params(params)
    io = st.io_torch

    # ---- training micro-batch (BASELINE config 3) --------------------------------------
    B, L = S.WORKLOADS["cfg3"]["train"]
    T = B * L
    X = S.normal_torch(0, "X", (B, L, d), 1.0, dev, io)
    dY = S.normal_torch(0, "dY", (B, L, d), S.WORKLOADS["cfg3"]["dy_std"], dev, io)
    Y = torch.empty_like(X)
    dX = torch.empty_like(X)
    dP = torch.zeros(st.ls_param_count(), dtype=torch.float32, device=dev)
    saved = st.new_saved(B, L)
    ws = st.new_workspace(T)

    def train():
        st.stage_train_fwd(X, B, L, Y, saved, ws)
        st.stage_train_bwd(dY, B, L, saved, dX, dP, 0, ws)

    # ---- serving batch (BASELINE config 4) -----------------------------------------------
    serve = S.WORKLOADS["cfg4"]["serve"]
    ctx = S.context_lengths(serve, seed=0)
    Bq = serve["B"]
    table, n_pages = S.page_tables(ctx, np.ones_like(ctx), P, seed=0)
    kv = Bd.KV(st, n_pages, table, ctx)
    kv.k_pool.copy_(S.normal_torch(0, "Kpool", kv.k_pool.shape, 1.0, dev, kv.k_pool.dtype))
    kv.v_pool.copy_(S.normal_torch(0, "Vpool", kv.v_pool.shape, 1.0, dev, kv.v_pool.dtype))
    Xd = S.normal_torch(0, "Xdec", (Bq, d), 1.0, dev, io)
    Yd = torch.empty_like(Xd)
    ws_a = st.new_workspace(max(Bq, 512))
    chunks = serve["prefill_chunks"]
    ptab, pn = S.page_tables(np.zeros(1, np.int64), np.array([sum(chunks)]), P, seed=1)
    kvp = [Bd.KV(st, pn, ptab, [0])]
    kvp.append(Bd.KV(st, pn, ptab, [chunks[0]]))
    kvp[1].k_pool, kvp[1].v_pool = kvp[0].k_pool, kvp[0].v_pool   # same pool, context advanced by chunk 0
    Xp = S.normal_torch(0, "Xprefill", (sum(chunks), d), 1.0, dev, io)
    Yp = torch.empty_like(Xp)

    # hybrid iteration-level mini-batch: the same 64 decode rows plus one 512-token prompt chunk in one call
    ctx_h = np.concatenate([ctx, np.zeros(1, ctx.dtype)])
    new_h = np.concatenate([np.ones_like(ctx), np.array([chunks[0]], ctx.dtype)])
    htab, hn = S.page_tables(ctx_h, new_h, P, seed=2)
    kvh = Bd.KV(st, hn, htab, ctx_h)
    kvh.k_pool.copy_(S.normal_torch(0, "Khyb", kvh.k_pool.shape, 1.0, dev, kvh.k_pool.dtype))
    kvh.v_pool.copy_(S.normal_torch(0, "Vhyb", kvh.v_pool.shape, 1.0, dev, kvh.v_pool.dtype))
    Xh = S.normal_torch(0, "Xhyb", (Bq + chunks[0], d), 1.0, dev, io)
    Yh = torch.empty_like(Xh)
    ws_h = st.new_workspace(Bq + chunks[0])

    def hybrid():
        st.stage_step(Xh, Bq, [chunks[0]], kvh, Yh, ws_h)

    def decode():
        st.stage_decode(Xd, Bq, kv, Yd, ws_a)

    def prefill():
        st.stage_prefill(Xp[:chunks[0]], [chunks[0]], kvp[0], Yp[:chunks[0]], ws_a)
        st.stage_prefill(Xp[chunks[0]:], [chunks[1]], kvp[1], Yp[chunks[0]:], ws_a)

    # ---- GEMM roofline: the 12 GEMM launches of one block, in the stage's own shapes -----------
    mt = Bd.TORCH_DTYPE[st.c.mma_dtype]
    U = 2 * F
    a_d = torch.randn(T, d, device=dev).to(mt)
    a_3d = torch.randn(T, 3 * d, device=dev).to(mt)
    a_U = torch.randn(T, U, device=dev).to(mt)
    a_F = torch.randn(T, F, device=dev).to(mt)
    w_qkv = (torch.randn(3 * d, d, device=dev) * 0.02).to(mt)
    w_o = (torch.randn(d, d, device=dev) * 0.02).to(mt)
    w_gu = (torch.randn(U, d, device=dev) * 0.02).to(mt)
    w_d = (torch.randn(d, F, device=dev) * 0.02).to(mt)
    o_3d, o_d, o_U, o_F = (torch.empty(T, n, device=dev, dtype=mt) for n in (3 * d, d, U, F))
    g_qkv, g_o, g_gu, g_d = (torch.empty_like(w, dtype=torch.float32) for w in (w_qkv, w_o, w_gu, w_d))
    G = Bd.lsk_gemm

    def gemms():
        G(a_d, w_qkv, o_3d, M=T, N=3 * d, K=d)
        G(a_d, w_o, o_d, M=T, N=d, K=d)
        G(a_d, w_gu, o_U, M=T, N=U, K=d)
        G(a_F, w_d, o_d, M=T, N=d, K=F)
        G(a_d, w_d, o_F, M=T, N=F, K=d, b_kmajor=False, ldb=F)
        G(a_d, a_F, g_d, M=d, N=F, K=T, a_kmajor=False, b_kmajor=False, lda=d, ldb=F)
        G(a_U, w_gu, o_d, M=T, N=d, K=U, b_kmajor=False, ldb=d)
        G(a_U, a_d, g_gu, M=U, N=d, K=T, a_kmajor=False, b_kmajor=False, lda=U, ldb=d)
        G(a_d, w_o, o_d, M=T, N=d, K=d, b_kmajor=False, ldb=d)
        G(a_d, a_d, g_o, M=d, N=d, K=T, a_kmajor=False, b_kmajor=False, lda=d, ldb=d)
        G(a_3d, w_qkv, o_d, M=T, N=d, K=3 * d, b_kmajor=False, ldb=d)
        G(a_3d, a_d, g_qkv, M=3 * d, N=d, K=T, a_kmajor=False, b_kmajor=False, lda=3 * d, ldb=d)

    # counter calibration: a plain copy kernel of known size (256 MiB read, 256 MiB written)
    cal_src = torch.zeros(64 << 20, dtype=torch.float32, device=dev)
    cal_dst = torch.empty_like(cal_src)

    def calib():
        Bd.lsk_convert(cal_src, cal_dst)

    legs = [l for l in args.legs.split(",") if l]
    leg_fn = {"train": train, "decode": decode, "prefill": prefill, "gemms": gemms, "calib": calib}
    leg_tok = {"train": T, "decode": Bq, "prefill": sum(chunks), "gemms": T, "calib": 0}

    def step():
        for l in legs:
            leg_fn[l]()

    tokens_per_step = sum(leg_tok[l] for l in legs)

    # ---- timed region: exactly K steps ------------------------------------------------------
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    log(f"step: {ms_per_step:.2f} ms")

    # ---- per-leg rates --------------------------------------------------------------------
    it = max(2, min(args.steps, 10))
    partial_run = set(legs) != {"train", "decode", "prefill"}
    ms_train = time_events(torch, train, it) if "train" in legs else float("nan")
    ms_dec = time_events(torch, decode, it * 2) if "decode" in legs else float("nan")
    ms_pre = time_events(torch, prefill, it) if "prefill" in legs else float("nan")
    if partial_run:
        print(json.dumps({"legs": legs, "ms_per_step": ms_per_step, "train_ms": ms_train, "decode_ms": ms_dec,
                          "prefill_ms": ms_pre}), flush=True)
        return
    ms_hyb = time_events(torch, hybrid, it)
    log(f"train {ms_train:.2f} ms, decode {ms_dec:.3f} ms, prefill {ms_pre:.2f} ms; hybrid 64 decode rows + one "
        f"512-token chunk in one call {ms_hyb:.2f} ms")

    # ---- GEMM roofline: the stage's own GEMM launches of the training leg, bracketed by HIP events inside the
    #      library (a pass of its own: the events add a few microseconds between launches) -----------------
    traffic = {}
    try:   # HBM bytes from rocprofv3 --pmc runs of this same command (see the file for command, date, commit)
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as fh:
            traffic = json.load(fh)
    except OSError:
        pass
    n_trace = 3
    train()
    torch.cuda.synchronize()
    Bd.lsk_timing_begin()
    for _ in range(n_trace):
        train()
    torch.cuda.synchronize()
    tr = Bd.lsk_timing_end()
    ms_g, n_g = tr["gemm"][0] / n_trace, tr["gemm"][1] // n_trace
    flop_gemm = 3.0 * T * nL * (8.0 * d * d + 6.0 * d * F)      # fwd + dX + dW of every block
    gemm_tflops = flop_gemm / (ms_g * 1e-3) / 1e12
    ms_gemms = time_events(torch, gemms, 5)                       # the same 12 shapes as bare lsk_gemm calls
    roofline = {"bound": "mfma", "kernel": "gemm_dma16_kernel (forward and input-gradient layouts) + gemm_dma_kernel<256,256> "
                "(weight gradients): the %d GEMM launches of stage_train_fwd + stage_train_bwd" % n_g,
                "achieved": gemm_tflops, "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": gemm_tflops / PEAK_MFMA_TFLOPS, "avg_launch_ms": ms_g / n_g, "launches_per_step": n_g,
                "flop_per_launch": flop_gemm / n_g, "measured": "HIP events around every GEMM launch of %d traced "
                "training steps (lsk_timing_begin / lsk_timing_end)" % n_trace,
                "traffic": traffic.get("gemm_bytes_per_launch", traffic.get("gemm_dma_kernel_bytes_per_launch")), "traffic_source": traffic.get("source"),
                "bare_gemm_calls_tflops": 3.0 * T * (8.0 * d * d + 6.0 * d * F) / (ms_gemms * 1e-3) / 1e12}
    train_kinds = {"gemm_ms": ms_g, "attention_fwd_ms": tr["attn_fwd"][0] / n_trace,
                   "attention_bwd_ms": tr["attn_bwd"][0] / n_trace}
    attn_flop_fwd = 2.0 * L * L * d * B * nL
    train_kinds["attention_fwd_tflops"] = attn_flop_fwd / (train_kinds["attention_fwd_ms"] * 1e-3) / 1e12
    train_kinds["attention_bwd_tflops"] = 2.0 * attn_flop_fwd / (train_kinds["attention_bwd_ms"] * 1e-3) / 1e12
    log(f"GEMMs of the training leg: {n_g} launches, {ms_g:.2f} ms -> {gemm_tflops:.0f} TFLOP/s "
        f"(bare calls of one block's 12 shapes: {roofline['bare_gemm_calls_tflops']:.0f}); attention fwd "
        f"{train_kinds['attention_fwd_ms']:.2f} ms, bwd {train_kinds['attention_bwd_ms']:.2f} ms")

    # ---- decode roofline: weights once + the KV of every cached token ---------------------------
    w_bytes = 2.0 * nL * (4.0 * d * d + 3.0 * d * F)
    kv_bytes = float((ctx + 1).sum()) * nL * 2 * d * 2
    dec_gbs = (w_bytes + kv_bytes) / (ms_dec * 1e-3) / 1e9
    decode()
    torch.cuda.synchronize()
    Bd.lsk_timing_begin()
    for _ in range(n_trace):
        decode()
    torch.cuda.synchronize()
    td = Bd.lsk_timing_end()
    dec_kinds = {k + "_ms": td[k][0] / n_trace for k in ("decode_attn", "decode_gemm", "finish")}
    dec_kinds["decode_attn_gbs"] = kv_bytes / (dec_kinds["decode_attn_ms"] * 1e-3) / 1e9
    dec_kinds["decode_gemm_gbs"] = w_bytes / (dec_kinds["decode_gemm_ms"] * 1e-3) / 1e9
    roofline_decode = {"bound": "hbm", "kernel": "stage_decode (whole call)", "achieved": dec_gbs,
                       "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": dec_gbs / PEAK_HBM_GBS,
                       "bytes_per_step": w_bytes + kv_bytes, "traffic": traffic.get("decode_step_bytes"),
                       "traffic_source": traffic.get("source"), "by_kind": dec_kinds}
    log(f"decode by kind: attention {dec_kinds['decode_attn_ms']:.3f} ms ({dec_kinds['decode_attn_gbs']:.0f} GB/s), "
        f"projections {dec_kinds['decode_gemm_ms']:.3f} ms ({dec_kinds['decode_gemm_gbs']:.0f} GB/s), "
        f"finish kernels {dec_kinds['finish_ms']:.3f} ms")

    # ---- interference probe (BASELINE config 4: decode stream + 1 x 2048 training stream) --------
    probe = None
    if not args.no_probe:
        Bt, Lt = S.WORKLOADS["cfg4"]["train"]
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        ms = st.stage_probe_interference(Xd, Bq, kv, Yd, ws_a, X[:Bt], Bt, Lt, Y[:Bt], saved, dY[:Bt],
                                         dX[:Bt], dP, ws, sa, sb, 3)
        torch.cuda.synchronize()
        probe = {"decode_alone_ms": ms[0], "train_alone_ms": ms[1], "decode_together_ms": ms[2],
                 "train_together_ms": ms[3], "wall_together_ms": ms[4],
                 "decode_tok_s_alone": Bq / ms[0] * 1e3, "decode_tok_s_together": Bq / ms[2] * 1e3,
                 "train_tok_s_alone": Bt * Lt / ms[1] * 1e3, "train_tok_s_together": Bt * Lt / ms[3] * 1e3}

    # ---- KV offload / reload of the longest request (PCIe-bound; reported, not part of the step) ------
    b_long = int(np.argmax(ctx))
    n_long = int(ctx[b_long])
    off_bytes = Bd.lsk_kv_packed_bytes(st, n_long)
    staging = torch.empty(off_bytes, dtype=torch.uint8, device=dev)
    hbuf = torch.empty(off_bytes, dtype=torch.uint8, pin_memory=True)
    ms_off = time_events(torch, lambda: Bd.lsk_kv_offload(st, kv, b_long, n_long, staging, hbuf), 3)
    ms_rel = time_events(torch, lambda: Bd.lsk_kv_reload(st, kv, b_long, n_long, hbuf, staging), 3)
    kv_move = {"request_tokens": n_long, "bytes": off_bytes, "offload_ms": ms_off, "reload_ms": ms_rel,
               "offload_gbs": off_bytes / (ms_off * 1e-3) / 1e9, "reload_gbs": off_bytes / (ms_rel * 1e-3) / 1e9,
               "note": "gather / scatter kernel plus one PCIe copy to / from pinned host memory"}
    log(f"KV offload of a {n_long}-token request ({off_bytes / 1e6:.0f} MB): {ms_off:.2f} ms out, {ms_rel:.2f} ms back")
    del staging, hbuf

    # ---- continuous-batching loop (Algorithm 3) over the same stage: 96 queued requests of 512 prompt
    #      tokens and 64 decode steps, C = 64, one hybrid mini-batch of at most 576 rows per pass ---------
    serve_loop = None
    if not args.no_serve_loop:
        from paper_2507_21276_amd import sched as Sc
        n_req, p_len, n_dec = 96, 512, 64
        pages_per_req = -(-(p_len + n_dec) // P)
        pool_shape = (nL, Bq * pages_per_req + 32, h, P, dh)
        kpl = torch.zeros(pool_shape, dtype=kv.k_pool.dtype, device=dev)
        vpl = torch.zeros_like(kpl)
        srv = Sc.Server(st, kpl, vpl, max_batch=Bq, max_wait=1e9, max_pages_per_req=pages_per_req,
                        max_chunk=p_len, max_tokens=Bq + p_len)
        Xr = S.normal_torch(0, "Xserve", (p_len + n_dec, d), 1.0, dev, io)
        Yr = [torch.empty_like(Xr) for _ in range(n_req)]
        for r in range(n_req):
            srv.submit(r, Xr, Yr[r], p_len, n_dec)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        passes = rows = 0
        host_s = 0.0
        while srv.in_flight():
            h0 = time.perf_counter()
            rep = srv.run_pass(time.perf_counter() - t0)
            host_s += time.perf_counter() - h0
            passes += 1
            rows += rep["n_rows"]
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        serve_loop = {"requests": n_req, "prompt_tokens": p_len, "decode_steps": n_dec, "max_batch": Bq,
                      "passes": passes, "rows": rows, "wall_ms": wall * 1e3, "rows_per_s": rows / wall,
                      "requests_per_s": n_req / wall, "ms_per_pass": wall * 1e3 / passes,
                      "pass_call_us": host_s * 1e6 / passes,
                      "pass_call_us_note": "wall time of one ls_server_pass call: host bookkeeping plus waiting for one "
                                           "of the two staging slots, i.e. for the GPU (the loop is GPU-bound)"}
        log(f"serve loop: {n_req} requests ({p_len} + {n_dec} rows) in {passes} passes, {wall * 1e3:.0f} ms "
            f"-> {rows / wall:.0f} rows/s ({host_s * 1e6 / passes:.0f} us per pass call, GPU-bound)")
        srv.close()
        del kpl, vpl, Yr

    # ---- BASELINE config 5 decode (LLaMA-13B-shaped stage, all ten blocks, 128 requests, lognormal contexts) ----
    decode_cfg5 = None
    if not args.no_cfg5:
        cfg5 = S.CONFIGS["llama13b_bf16"]
        st5 = Bd.Stage(cfg5, io_dtype="bf16", mma_dtype=args.mma)
        p5 = S.make_params_torch(cfg5, seed=0, device=dev)
        st5.ls_bind_params(p5)
        sv5 = S.WORKLOADS["cfg5"]["serve"]
        ctx5 = S.context_lengths(sv5, seed=0)
        B5, d5, F5, nL5 = sv5["B"], cfg5["d_model"], cfg5["d_ff"], cfg5["n_layers"]
        tab5, np5 = S.page_tables(ctx5, np.ones_like(ctx5), cfg5["page_size"], seed=0)
        kv5 = Bd.KV(st5, np5, tab5, ctx5)
        kv5.k_pool.copy_(S.normal_torch(0, "Kpool5", kv5.k_pool.shape, 1.0, dev, kv5.k_pool.dtype))
        kv5.v_pool.copy_(S.normal_torch(0, "Vpool5", kv5.v_pool.shape, 1.0, dev, kv5.v_pool.dtype))
        X5 = S.normal_torch(0, "Xdec5", (B5, d5), 1.0, dev, io)
        Y5 = torch.empty_like(X5)
        ws5 = st5.new_workspace(B5)
        ms5 = time_events(torch, lambda: st5.stage_decode(X5, B5, kv5, Y5, ws5), 10, warm=2)
        by5 = 2.0 * nL5 * (4.0 * d5 * d5 + 3.0 * d5 * F5) + float((ctx5 + 1).sum()) * nL5 * 2 * d5 * 2
        decode_cfg5 = {"workload": "cfg5 decode B=128 ctx~lognormal(median 1024) clipped [64, 4096], 10 blocks",
                       "ms": ms5, "tok_s": B5 / ms5 * 1e3, "bytes": by5, "achieved_gbs": by5 / (ms5 * 1e-3) / 1e9,
                       "frac_of_hbm_peak": by5 / (ms5 * 1e-3) / 1e9 / PEAK_HBM_GBS}
        log(f"cfg5 decode (10 blocks): {ms5:.2f} ms -> {decode_cfg5['achieved_gbs']:.0f} GB/s")
        st5.close()
        del kv5, p5, X5, Y5, ws5

    # ---- the other operand format: the same training and decode legs on a stage with bf16 (default fp16)
    #      matrix-core operands, and the other way round under --mma bf16 -----------------------------------
    other_mode = None
    if not args.no_other_mode:
        om = "bf16" if args.mma == "f16" else "f16"
        st2 = Bd.Stage(cfg, io_dtype="bf16", mma_dtype=om)
        st2.ls_bind_params(params)
        kv2 = Bd.KV(st2, n_pages, table, ctx)
        kv2.k_pool.copy_(kv.k_pool.to(kv2.k_pool.dtype))
        kv2.v_pool.copy_(kv.v_pool.to(kv2.v_pool.dtype))

        def train2():
            st2.stage_train_fwd(X, B, L, Y, saved, ws)
            st2.stage_train_bwd(dY, B, L, saved, dX, dP, 0, ws)

        ms_t2 = time_events(torch, train2, 5)
        ms_d2 = time_events(torch, lambda: st2.stage_decode(Xd, Bq, kv2, Yd, ws_a), 10)
        Bd.lsk_timing_begin()
        train2()
        torch.cuda.synchronize()
        t2 = Bd.lsk_timing_end()
        other_mode = {"mma_operands": om, "train_ms": ms_t2, "train_tok_s": T / ms_t2 * 1e3, "decode_ms": ms_d2,
                      "gemm_tflops": flop_gemm / (t2["gemm"][0] * 1e-3) / 1e12,
                      "gemm_frac_of_mfma_peak": flop_gemm / (t2["gemm"][0] * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS}
        log(f"{om} operands: train {ms_t2:.2f} ms, decode {ms_d2:.3f} ms, GEMMs {other_mode['gemm_tflops']:.0f} TFLOP/s")
        st2.close()
        del kv2

    # ---- model update (a row beyond the step: AdamW over the stage's parameters, last because it
    #      rewrites the weights) -------------------------------------------------------------------
    roofline_update = None
    if not args.no_update:
        n_par = st.ls_param_count()
        master = params.to(torch.float32)
        m_buf = torch.zeros(n_par, dtype=torch.float32, device=dev)
        v_buf = torch.zeros(n_par, dtype=torch.float32, device=dev)
        step_no = [0]

        def update():
            step_no[0] += 1
            st.stage_optimizer_step(params, master, m_buf, v_buf, dP, kind=Bd.LS_OPT_ADAMW, lr=1e-5,
                                    step=step_no[0], weight_decay=0.01)

        ms_upd = time_events(torch, update, 3)
        upd_bytes = 32.0 * n_par    # g, m, v, w read; m, v, w written; bf16 parameter and fp16 operand copy written
        roofline_update = {"bound": "hbm", "kernel": "optimizer_kernel (AdamW, fused refresh of the bf16 parameters "
                           "and the fp16 operand copy)", "achieved": upd_bytes / (ms_upd * 1e-3) / 1e9,
                           "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": upd_bytes / (ms_upd * 1e-3) / 1e9 / PEAK_HBM_GBS, "ms": ms_upd,
                           "bytes_per_step": upd_bytes, "traffic": None}
        log(f"model update: {ms_upd:.2f} ms -> {roofline_update['achieved']:.0f} GB/s")
        del master, m_buf, v_buf

    out = {
        "metric": "stage tok/s (train fwd+bwd + ragged decode + prefill chunks), LLaMA-7B-shaped 8-block stage, 1 MI355X",
        "value": tokens_per_step / (ms_per_step * 1e-3), "unit": "tok/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": f"{args.mma} MFMA operands, bf16 parameters and io, fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": "cfg3 train 2x2048 fwd+bwd + cfg4 ragged decode B=64 ctx~U[128,2048] paged(16) "
                               "+ cfg4 prefill 2x512", "stage": "llama7b_bf16", "n_layers": nL, "d_model": d,
                   "d_ff": F, "tokens_per_step": tokens_per_step},
        "breakdown": {"train_fwd_bwd_tok_s": T / ms_train * 1e3, "train_ms": ms_train,
                      "decode_tok_s": Bq / ms_dec * 1e3, "decode_ms": ms_dec,
                      "prefill_tok_s": sum(chunks) / ms_pre * 1e3, "prefill_ms": ms_pre,
                      "hybrid_decode64_chunk512_ms": ms_hyb,
                      "hybrid_separate_calls_ms": ms_dec + ms_pre / len(chunks),
                      "train_frac_of_mfma_peak": (3.0 * T * nL * (8.0 * d * d + 6.0 * d * F)
                                                  + 3.0 * 2.0 * L * L * d * B * nL) / (ms_train * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS},
        "roofline": roofline, "roofline_decode": roofline_decode, "roofline_update": roofline_update,
        "train_by_kind": train_kinds, "other_operand_format": other_mode,
        "probe": probe, "kv_offload": kv_move, "serve_loop": serve_loop, "decode_cfg5": decode_cfg5,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, S)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
