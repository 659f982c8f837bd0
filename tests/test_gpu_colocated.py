"""Co-located run of one stage on the GPU, driven by the library's own host steps: training and
inference tasks are planned on a node (Algorithm 1), executed in queue order by the memory-aware
loop (Algorithm 2) whose hooks are the real stage calls, inference tasks go through the
continuous-batching server (Algorithm 3), and every training task ends with a model update.
Checked against the float64 oracle: each task computes with the weights that the updates before
it left behind, which is the paper's on-the-fly adaptation."""
import time

import numpy as np
import pytest
import torch

from oracle import sched_oracle as SO
from oracle import stage_oracle as O
from paper_2507_21276_amd import binding as Bd
from paper_2507_21276_amd import sched as Sc
from paper_2507_21276_amd import synth_inputs as S
from parity_util import TOL, assert_close, dev, host

pytestmark = pytest.mark.gpu

CFG = S.scaled(S.CONFIGS["llama7b_bf16"], n_layers=2, d_model=256, n_heads=2, d_ff=704)
SGD = dict(lr=2e-2, weight_decay=0.0, momentum=0.0, grad_scale=1.0)


def test_training_and_inference_tasks_through_the_memory_aware_loop():
    cfg = CFG
    d, P = cfg["d_model"], cfg["page_size"]
    st = Bd.Stage(cfg, io_dtype="f32", mma_dtype="f16")
    flat = S.make_params(cfg, seed=0, perturb_norm=0.1)
    n = flat.size
    pd = dev(flat, st.param_torch)
    st.ls_bind_params(pd)
    master = dev(flat, torch.float32)
    mom = torch.zeros(n, dtype=torch.float32, device="cuda")
    dP = torch.empty(n, dtype=torch.float32, device="cuda")

    # tasks in arrival order: (kind, arrival, ...)
    B, L = 2, 48
    tasks = [("train", 0.00), ("serve", 0.01, 40, 4), ("train", 0.02), ("serve", 0.03, 24, 3), ("serve", 0.03, 70, 0)]
    node = Sc.Node(1, 1e-7, 2e-7)
    node_ref = SO.Node(1, 1e-7, 2e-7)
    data, ids = {}, []
    for i, t in enumerate(tasks):
        if t[0] == "train":
            X = S.make_activations(cfg, f"X{i}", (B, L, d))
            dY = S.make_activations(cfg, f"dY{i}", (B, L, d))
            data[i] = dict(X=X, dY=dY, Y=torch.empty(B, L, d, dtype=st.io_torch, device="cuda"))
            p = node.plan(t[1], L, B, True, commit=True)
            SO.commit(node_ref, t[1], L, B, True)
        else:
            X = S.make_activations(cfg, f"Xs{i}", (t[2] + t[3], d))
            data[i] = dict(X=X, Xd=dev(X, st.io_torch), Y=torch.zeros(t[2] + t[3], d, dtype=st.io_torch, device="cuda"))
            p = node.plan(t[1], t[2], 1, False, commit=True)
            SO.commit(node_ref, t[1], t[2], 1, False)
        ids.append(p["id"])
    assert ids == list(range(len(tasks))) and node.queue_len() == len(tasks)
    assert node.queue_len(True) == len(node_ref.train)

    n_pages = 16
    shape = (cfg["n_layers"], n_pages, cfg["n_heads"], P, cfg["head_dim"])
    kp = torch.zeros(shape, dtype=torch.float16, device="cuda")
    vp = torch.zeros_like(kp)
    srv = Sc.Server(st, kp, vp, max_batch=4, max_wait=10.0, max_pages_per_req=8, max_chunk=32, max_tokens=64)
    ws, saved = st.new_workspace(B * L), st.new_saved(B, L)
    dX = torch.empty(B, L, d, dtype=st.io_torch, device="cuda")
    t0 = time.perf_counter()
    weights_seen, log, mem_checks = {}, [], []

    def now():
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def memory_available(stage):
        need = st.ls_saved_bytes(B, L) + st.ls_workspace_bytes(B * L)
        ok, used = Bd.lsk_memory_available(need, 250 << 30)
        mem_checks.append(ok)
        return ok

    def forward(tid, stage):
        a = now()
        weights_seen[tid] = host(pd)          # the stored weights this task computes with
        t = tasks[tid]
        if t[0] == "train":
            st.stage_train_fwd(dev(data[tid]["X"], st.io_torch), B, L, data[tid]["Y"], saved, ws)
        else:
            q = data[tid]
            srv.submit(tid, q["Xd"], q["Y"], t[2], t[3])
            passes = 0
            while srv.in_flight():
                rep = srv.run_pass(now())
                assert rep["n_rows"] > 0
                passes += 1
            log.append(("serve", tid, passes))
        return a, now()

    def backward(tid):
        a = now()
        st.stage_train_bwd(dev(data[tid]["dY"], st.io_torch), B, L, saved, dX, dP, 0, ws)
        data[tid]["dP"] = host(dP)
        st.stage_optimizer_step(pd, master, mom, None, dP, kind=Bd.LS_OPT_SGD, step=1, **SGD)
        b = now()
        log.append(("update", tid))
        return [a], [b]

    stats = node.execute(0.001, 0.01, memory_available, lambda s: None, lambda tid, s: log.append(("offload", tid)),
                         forward, backward)
    torch.cuda.synchronize()
    assert stats["tasks"] == 5 and stats["forwards"] == 5 and stats["backwards"] == 2 and stats["offloads"] == 0
    assert all(mem_checks) and len(mem_checks) == 10          # loop test and the test before Forward, per task
    assert [e for e in log if e[0] == "update"] == [("update", 0), ("update", 2)]
    # prompt of 40 in chunks of 32 + 8, then 4 decode passes; 24 -> 1 + 3; 70 -> 32 + 32 + 6
    assert [e for e in log if e[0] == "serve"] == [("serve", 1, 6), ("serve", 3, 4), ("serve", 4, 3)]

    # calibrated paths: measured intervals, in execution order
    ends = 0.0
    for tid in ids:
        p = node.path(tid)
        assert p["start_f"][0] >= ends - 1e-9 and p["end_f"][0] > p["start_f"][0]
        ends = p["end_f"][0]
        if tasks[tid][0] == "train":
            assert p["start_b"][0] >= p["end_f"][0] - 1e-9 and p["end_b"][0] > p["start_b"][0]
            ends = p["end_b"][0]

    # numerics: every task against the oracle with the weights it saw; the updates against the oracle's rule
    tol = TOL["bf16"]
    w_before = flat.astype(np.float64)
    for tid in ids:
        w = weights_seen[tid]
        t = tasks[tid]
        if t[0] == "train":
            Yr, sv = O.stage_train_fwd(cfg, w, data[tid]["X"].astype(np.float64))
            assert_close(host(data[tid]["Y"]), Yr, tol, f"training forward of task {tid}")
            wr, _, _ = O.optimizer_step("sgd", w_before, data[tid]["dP"], np.zeros(n), np.zeros(n), 1,
                                        decay=O.decay_mask(cfg), **SGD)
            w_before = wr          # fp32 master after this update (the oracle's, from the GPU's own gradients)
        else:
            ref = O.stage_prefill(cfg, w, [data[tid]["X"].astype(np.float64)], O.new_cache(cfg, 1))[0]
            assert_close(host(data[tid]["Y"]), ref, tol, f"inference task {tid}")
    assert_close(host(master), w_before, 1e-5, "master weights after both updates")
    # the three inference tasks ran on three different sets of weights (after update 1, after update 2 twice)
    assert not np.array_equal(weights_seen[1], weights_seen[0])
    assert not np.array_equal(weights_seen[3], weights_seen[1]) and np.array_equal(weights_seen[3], weights_seen[4])
    srv.close()
    st.close()
