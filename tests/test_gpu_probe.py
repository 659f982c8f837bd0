"""Co-located execution on one GPU (System Model; Motivation, the interference study): a decode
step on one stream and a training forward + backward on another, enqueued together.

What is checked: the results of the two tasks when they run concurrently - through
stage_probe_interference and enqueued directly on two streams - are bit-identical to the results
of the same calls run alone (Y of the decode step, the K/V rows it writes, Y, dX and every
parameter gradient of the training task), and both are within tolerance of the float64 oracle.
"""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import stage_oracle as O
from paper_2507_21276_amd import binding as Bd
from paper_2507_21276_amd import synth_inputs as S
from parity_util import TOL, assert_close, dev, host, out_rounding_bound, param_slices

pytestmark = pytest.mark.gpu

SMALL_LLAMA = S.scaled(S.CONFIGS["llama7b_bf16"], n_layers=2, d_model=256, n_heads=2, d_ff=688)
SMALL_GPT = S.scaled(S.CONFIGS["gpt2s_bf16"], n_layers=2, d_model=256, n_heads=4, d_ff=1024)


class Colocated:
    """One decode batch over a seeded cache and one training micro-batch on the same stage."""

    def __init__(self, cfg, ctx, B, L, io, dy_std, seed=0):
        self.cfg, self.B, self.L = cfg, B, L
        d, P = cfg["d_model"], cfg["page_size"]
        self.st = st = Bd.Stage(cfg, io_dtype=io, mma_dtype="f16")
        self.pd = S.make_params_torch(cfg, seed=seed)
        st.ls_bind_params(self.pd)
        self.ctx = np.asarray(ctx, np.int64)
        self.Bq = len(self.ctx)
        self.table, n_pages = S.page_tables(self.ctx, np.ones_like(self.ctx), P, seed=seed)
        self.kv = kv = Bd.KV(st, n_pages, self.table, self.ctx)
        kv.k_pool.copy_(S.normal_torch(seed, "Kpool", kv.k_pool.shape, 1.0, "cuda", kv.k_pool.dtype))
        kv.v_pool.copy_(S.normal_torch(seed, "Vpool", kv.v_pool.shape, 1.0, "cuda", kv.v_pool.dtype))
        self.pool0 = (kv.k_pool.clone(), kv.v_pool.clone())
        bf = torch.bfloat16
        self.Xdec = S.normal_torch(seed, "Xdec", (self.Bq, d), 1.0, "cuda", bf).to(st.io_torch)
        self.X = S.normal_torch(seed, "X", (B, L, d), 1.0, "cuda", bf).to(st.io_torch)
        self.dY = S.normal_torch(seed, "dY", (B, L, d), dy_std, "cuda", bf).to(st.io_torch)
        self.ws_a, self.ws_b = st.new_workspace(self.Bq), st.new_workspace(B * L)
        self.saved = st.new_saved(B, L)
        self.sa, self.sb = torch.cuda.Stream(), torch.cuda.Stream()
        self.fresh_outputs()

    def fresh_outputs(self):
        """Outputs refilled with a marker and the pools restored, so that a call that wrote nothing shows."""
        self.Ydec = torch.full_like(self.Xdec, 7.0)
        self.Y, self.dX = torch.full_like(self.X, 7.0), torch.full_like(self.X, 7.0)
        self.dP = torch.full((self.st.ls_param_count(),), 7.0, dtype=torch.float32, device="cuda")
        self.kv.k_pool.copy_(self.pool0[0])
        self.kv.v_pool.copy_(self.pool0[1])
        torch.cuda.synchronize()

    def decode(self, stream):
        self.st.stage_decode(self.Xdec, self.Bq, self.kv, self.Ydec, self.ws_a, stream=stream)

    def train(self, stream):
        self.st.stage_train_fwd(self.X, self.B, self.L, self.Y, self.saved, self.ws_b, stream=stream)
        self.st.stage_train_bwd(self.dY, self.B, self.L, self.saved, self.dX, self.dP, 0, self.ws_b, stream=stream)

    def snapshot(self):
        torch.cuda.synchronize()
        return {"Ydec": self.Ydec.clone(), "k_pool": self.kv.k_pool.clone(), "v_pool": self.kv.v_pool.clone(),
                "Y": self.Y.clone(), "dX": self.dX.clone(), "dP": self.dP.clone()}

    def alone(self):
        self.fresh_outputs()
        self.decode(self.sa)
        torch.cuda.synchronize()
        self.train(self.sb)
        return self.snapshot()

    def together_direct(self, decode_steps):
        """The training task is enqueued first (it is the long one); decode steps keep arriving on the
        other stream while it runs.  ctx_len is not advanced, so every step rewrites the same rows."""
        self.fresh_outputs()
        self.train(self.sb)
        for _ in range(decode_steps):
            self.decode(self.sa)
        return self.snapshot()

    def together_probe(self, iters):
        self.fresh_outputs()
        ms = self.st.stage_probe_interference(self.Xdec, self.Bq, self.kv, self.Ydec, self.ws_a, self.X, self.B, self.L,
                                              self.Y, self.saved, self.dY, self.dX, self.dP, self.ws_b, self.sa, self.sb,
                                              iters)
        return self.snapshot(), ms

    def oracle(self):
        cfg, P = self.cfg, self.cfg["page_size"]
        flat = host(self.pd)
        kp, vp = self.pool0[0].float().cpu().numpy(), self.pool0[1].float().cpu().numpy()
        cache = []
        for l in range(cfg["n_layers"]):
            per = []
            for b, c in enumerate(self.ctx):
                j = np.arange(int(c))
                pg = self.table[b, j // P]
                per.append([kp[l, pg, :, j % P, :].astype(np.float64), vp[l, pg, :, j % P, :].astype(np.float64)])
            cache.append(per)
        Ydec = O.stage_decode(cfg, flat, host(self.Xdec), cache)
        Y, sv = O.stage_train_fwd(cfg, flat, host(self.X))
        dX, dP = O.stage_train_bwd(cfg, flat, sv, host(self.dY))
        return {"Ydec": Ydec, "cache": cache, "Y": Y, "dX": dX, "dP": dP}

    def close(self):
        self.st.close()


def assert_bit_identical(got, ref, what):
    for k in ref:
        assert torch.equal(got[k], ref[k]), f"{what}: {k} differs from the run alone"


def check_against_oracle(case, snap, io):
    cfg, P = case.cfg, case.cfg["page_size"]
    ref = case.oracle()
    tol = TOL["bf16"]

    def bar(r):    # results that leave the stage in bf16 carry their own rounding (half an ulp of the largest element)
        return tol + (out_rounding_bound(r, "bf16") if io == "bf16" else 0.0)

    errs = {k: assert_close(host(snap[k]), ref[k], bar(ref[k]), k) for k in ("Ydec", "Y", "dX")}
    dP = host(snap["dP"])
    for name, off, n in param_slices(cfg):
        errs[name] = assert_close(dP[off:off + n], ref["dP"][off:off + n], tol, "grad " + name)
    # the K / V rows the decode step appended, every block, every request
    kp, vp = snap["k_pool"].float().cpu().numpy(), snap["v_pool"].float().cpu().numpy()
    for l in range(cfg["n_layers"]):
        K = np.stack([kp[l, case.table[b, c // P], :, c % P, :] for b, c in enumerate(case.ctx)])
        V = np.stack([vp[l, case.table[b, c // P], :, c % P, :] for b, c in enumerate(case.ctx)])
        Kr = np.stack([ref["cache"][l][b][0][int(c)] for b, c in enumerate(case.ctx)])
        Vr = np.stack([ref["cache"][l][b][1][int(c)] for b, c in enumerate(case.ctx)])
        assert_close(K, Kr, tol, f"new K rows, block {l}")
        assert_close(V, Vr, tol, f"new V rows, block {l}")
    # and nothing else in the pools moved
    untouched = torch.ones(kp.shape[1], P, dtype=torch.bool)
    for b, c in enumerate(case.ctx):
        untouched[case.table[b, c // P], c % P] = False
    m = untouched.cuda()[None, :, None, :, None].expand_as(snap["k_pool"])
    assert torch.equal(snap["k_pool"][m], case.pool0[0][m]) and torch.equal(snap["v_pool"][m], case.pool0[1][m])
    return errs


@pytest.mark.parametrize("which", ["llama", "gpt"])
def test_decode_and_training_run_together_as_they_run_alone_small_stage(which):
    cfg = SMALL_LLAMA if which == "llama" else SMALL_GPT
    ctx = [0, 1, 15, 16, 17, 100, 333, 257, 64, 31]
    case = Colocated(cfg, ctx, 2, 200, io="f32", dy_std=1e-2 if which == "llama" else 1.0)
    alone = case.alone()
    for k in ("Ydec", "Y", "dX", "dP"):
        assert not (alone[k] == 7.0).all(), k + " was not written"
    assert_bit_identical(case.together_direct(decode_steps=12), alone, "two streams, enqueued directly")
    snap, ms = case.together_probe(iters=3)
    assert_bit_identical(snap, alone, "stage_probe_interference")
    assert all(v > 0 for v in ms[:5]) and ms[5] == 0
    assert ms[4] >= max(ms[2], ms[3]) * 0.95       # the wall time of a round covers both streams
    check_against_oracle(case, alone, "f32")
    case.close()


def test_decode_and_training_run_together_cfg4_shapes_two_blocks():
    """Config 4's own shapes and element types (ragged decode batch of 64, 1 x 2048 training micro-batch, bf16
    io as the benchmark builds it); two of the eight blocks keep the float64 oracle to seconds."""
    cfg = S.scaled(S.CONFIGS["llama7b_bf16"], n_layers=2)
    wl = S.WORKLOADS["cfg4"]
    ctx = S.context_lengths(wl["serve"])
    B, L = wl["train"]
    case = Colocated(cfg, ctx, B, L, io="bf16", dy_std=wl["dy_std"])
    alone = case.alone()
    assert_bit_identical(case.together_direct(decode_steps=8), alone, "two streams, enqueued directly")
    snap, ms = case.together_probe(iters=2)
    assert_bit_identical(snap, alone, "stage_probe_interference")
    assert ms[2] >= ms[0] * 0.8 and ms[3] >= ms[1] * 0.8   # sharing the GPU does not make either task faster
    errs = check_against_oracle(case, alone, "bf16")
    print("cfg4 co-located, worst error", max(errs.items(), key=lambda kv: kv[1]))
    case.close()


def test_probe_rejects_bad_arguments():
    case = Colocated(SMALL_LLAMA, [5, 40], 1, 64, io="f32", dy_std=1e-2)
    st, out = case.st, (C.c_float * 6)()
    d = case.kv.desc(True)

    def call(ws_a, ws_b, sa, sb, iters, out_ms=out, dec_B=case.Bq):
        return Bd.lib().stage_probe_interference(
            st.h, case.Xdec.data_ptr(), dec_B, C.byref(d), case.Ydec.data_ptr(), ws_a, case.X.data_ptr(), case.B,
            case.L, case.Y.data_ptr(), case.saved.data_ptr(), case.dY.data_ptr(), case.dX.data_ptr(),
            case.dP.data_ptr(), ws_b, sa, sb, iters, out_ms)

    a, b = case.ws_a.data_ptr(), case.ws_b.data_ptr()
    sa, sb = case.sa.cuda_stream, case.sb.cuda_stream
    assert call(a, b, sa, sa, 1) == Bd.LS_EINVAL and b"streams" in Bd.lib().ls_last_error()
    assert call(a, a, sa, sb, 1) == Bd.LS_EINVAL and b"workspaces" in Bd.lib().ls_last_error()
    assert call(a, b, sa, sb, 0) == Bd.LS_EINVAL
    assert call(a, b, sa, sb, 1, out_ms=None) == Bd.LS_EINVAL
    assert call(a, b, sa, sb, 1, dec_B=0) == Bd.LS_EINVAL
    assert call(a, b, sa, sb, 1) == Bd.LS_OK
    case.close()
