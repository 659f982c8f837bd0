"""The continuous-batching loop on the GPU (ls_server_*) against the oracles: which rows run
in which pass (bit-exact against the bookkeeping model) and every request's output rows
(against the float64 stage forward over the request's whole sequence, which is what prompt
chunks plus cached decode steps compute)."""
import numpy as np
import pytest
import torch

from oracle import stage_oracle as O
from oracle.serve_oracle import ServeModel
from paper_2507_21276_amd import binding as Bd
from paper_2507_21276_amd import sched as Sc
from paper_2507_21276_amd import synth_inputs as S
from parity_util import TOL, assert_close, dev, host

pytestmark = pytest.mark.gpu

SMALL_LLAMA = S.scaled(S.CONFIGS["llama7b_bf16"], n_layers=2, d_model=256, n_heads=2, d_ff=688)
TINY = S.CONFIGS["tiny_gpt_f32"]


def run_trace(cfg, mma, *, C, T_w, n_pages, max_chunk, max_tokens, n_req, seed, max_prompt, max_decode, min_prompt=1, expect_hybrid=True):
    rng = np.random.default_rng(seed)
    io = "f32" if cfg["dtype"] == "bf16" else None
    st = Bd.Stage(cfg, io_dtype=io, mma_dtype=mma)
    flat = S.make_params(cfg, seed=0, perturb_norm=0.1)
    st.ls_bind_params(dev(flat, st.param_torch))
    d, P = cfg["d_model"], cfg["page_size"]
    max_pages = -(-(max_prompt + max_decode) // P)
    shape = (cfg["n_layers"], n_pages, cfg["n_heads"], P, cfg["head_dim"])
    kp = torch.zeros(shape, dtype=Bd.TORCH_DTYPE[st.c.mma_dtype], device="cuda")
    vp = torch.zeros_like(kp)
    srv = Sc.Server(st, kp, vp, max_batch=C, max_wait=T_w, max_pages_per_req=max_pages, max_chunk=max_chunk,
                    max_tokens=max_tokens)
    model = ServeModel(C, T_w, n_pages, P, max_chunk, max_tokens)
    reqs, arrivals = {}, {}
    for r in range(n_req):
        pl, nd = int(rng.integers(min_prompt, max_prompt + 1)), int(rng.integers(0, max_decode + 1))
        X = S.make_activations(cfg, f"Xreq{r}", (pl + nd, d))
        reqs[r] = dict(X=X, Xd=dev(X, st.io_torch), Y=torch.zeros(pl + nd, d, dtype=st.io_torch, device="cuda"),
                       pl=pl, nd=nd)
        arrivals.setdefault(int(rng.integers(0, n_req)), []).append(r)
    now, it, finished, rows_total, hybrid_passes = 0.0, 0, [], 0, 0
    while it < n_req or srv.in_flight():
        for r in arrivals.get(it, []):
            q = reqs[r]
            srv.submit(r, q["Xd"], q["Y"], q["pl"], q["nd"])
            model.submit(r, q["pl"], q["nd"])
        rep = srv.run_pass(now)
        members, fin, _, nb, nn = model.run_pass(now)
        assert rep["ran"] == [m[0] for m in members], (it, rep, members)
        assert rep["finished"] == fin and rep["n_batch"] == nb and rep["n_new"] == nn
        assert rep["n_rows"] == sum(m[2] for m in members)
        assert rep["n_decode"] == sum(m[1] >= reqs[m[0]]["pl"] for m in members)
        assert rep["free_pages"] == len(model.free) and rep["unreserved_pages"] == model.unreserved
        assert rep["n_rows"] > 0 or nb == 0, "a pass with members in the batch made no progress"
        hybrid_passes += rep["n_decode"] > 0 and rep["n_prefill"] > 0
        finished += fin
        rows_total += rep["n_rows"]
        now += float(rng.exponential(0.02))
        it += 1
        assert it < 50 * n_req, "the loop does not drain"
    torch.cuda.synchronize()
    assert sorted(finished) == list(range(n_req)) and rows_total == sum(q["pl"] + q["nd"] for q in reqs.values())
    assert hybrid_passes > 0 or not expect_hybrid
    f64 = flat.astype(np.float64)
    tol = TOL["bf16"] if mma else TOL["f32"]
    worst = 0.0
    for r, q in reqs.items():
        cache = O.new_cache(cfg, 1)
        ref = O.stage_prefill(cfg, f64, [q["X"].astype(np.float64)], cache)[0]
        worst = max(worst, assert_close(host(q["Y"]), ref, tol, f"request {r} ({q['pl']} + {q['nd']} rows)"))
    srv.close()
    st.close()
    return worst


def test_serve_loop_small_llama_f16():
    # pool too small for everything at once (members wait for pages), chunked prompts, row budget
    worst = run_trace(SMALL_LLAMA, "f16", C=6, T_w=0.05, n_pages=20, max_chunk=48, max_tokens=96, n_req=24,
                      seed=5, max_prompt=150, max_decode=12)
    print(f"serve loop, small llama f16: worst relative error {worst:.2e}")


def test_serve_loop_drains_when_the_pool_is_smaller_than_the_batch_members_need_together():
    """Six members of up to eleven pages each over a pool of twelve pages, with a row budget large enough for
    all of them to start at once: without setting a request's pages aside at its start every member would hold
    part of its pages and none could finish.  Every pass must make progress, and the rows must still be right."""
    worst = run_trace(SMALL_LLAMA, "f16", C=6, T_w=0.05, n_pages=12, max_chunk=48, max_tokens=288, n_req=18,
                      seed=11, max_prompt=150, max_decode=12, min_prompt=100, expect_hybrid=False)
    print(f"serve loop, pool of 12 pages: worst relative error {worst:.2e}")


def test_serve_loop_widths_that_take_the_fused_decode_path():
    # d_ff a multiple of 64 and at most 128 rows per pass: every pass (decode rows, prompt chunks, or both)
    # runs the partial-product projections and the fused finish kernels
    cfg = S.scaled(S.CONFIGS["llama7b_bf16"], n_layers=3, d_model=256, n_heads=2, d_ff=704)
    worst = run_trace(cfg, "f16", C=8, T_w=0.05, n_pages=40, max_chunk=64, max_tokens=128, n_req=20,
                      seed=7, max_prompt=200, max_decode=10)
    print(f"serve loop, fused decode path: worst relative error {worst:.2e}")


def test_serve_loop_tiny_gpt_f32():
    worst = run_trace(TINY, None, C=4, T_w=0.03, n_pages=24, max_chunk=16, max_tokens=40, n_req=16, seed=6,
                      max_prompt=40, max_decode=8)
    print(f"serve loop, tiny gpt fp32: worst relative error {worst:.2e}")


def test_serve_loop_argument_errors():
    st = Bd.Stage(TINY)
    st.ls_bind_params(dev(S.make_params(TINY, seed=0), st.param_torch))
    P = TINY["page_size"]
    shape = (TINY["n_layers"], 4, TINY["n_heads"], P, TINY["head_dim"])
    kp = torch.zeros(shape, device="cuda")
    vp = torch.zeros_like(kp)
    with pytest.raises(Bd.LsError):
        Sc.Server(st, kp, vp, max_batch=0, max_wait=0.1, max_pages_per_req=2, max_chunk=8, max_tokens=16)
    with pytest.raises(Bd.LsError):
        Sc.Server(st, kp, vp, max_batch=8, max_wait=0.1, max_pages_per_req=2, max_chunk=8, max_tokens=4)
    srv = Sc.Server(st, kp, vp, max_batch=2, max_wait=0.1, max_pages_per_req=2, max_chunk=8, max_tokens=16)
    X = torch.zeros(3 * P, TINY["d_model"], device="cuda")
    with pytest.raises(Bd.LsError):
        srv.submit(0, X, X, 2 * P, 1)            # more tokens than max_pages_per_req pages hold
    with pytest.raises(Bd.LsError):
        srv.submit(0, X, X, 0, 1)                # empty prompt
    srv.submit(0, X, X, 4, 1)
    with pytest.raises(Bd.LsError):
        srv.submit(0, X, X, 4, 1)                # id already in flight
    rep = srv.run_pass(0.0)
    assert rep["ran"] == [0] and rep["n_rows"] == 4
    torch.cuda.synchronize()
    srv.close()
    st.close()
