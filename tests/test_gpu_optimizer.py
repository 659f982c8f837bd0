"""GPU parity of the model-update kernel and of serving from updated weights (through the C ABI).

Bar: fp32 arithmetic against the float64 oracle, max-abs error over RMS <= 1e-5 for the master
weights and both moments after several steps; the 16-bit copies are bit-exact roundings of what
the kernel itself holds in fp32.
"""
import numpy as np
import pytest
import torch

from oracle import stage_oracle as O
from paper_2507_21276_amd import binding as Bd
from paper_2507_21276_amd import synth_inputs as S
from parity_util import TOL, assert_close, dev, host
from test_gpu_stage import SMALL_GPT, SMALL_LLAMA, make_stage

pytestmark = pytest.mark.gpu

HYPER = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-6, weight_decay=0.1, momentum=0.8, grad_scale=0.5)


def oracle_kwargs(kind):
    return dict(HYPER) if kind == "adamw" else dict(lr=HYPER["lr"], weight_decay=HYPER["weight_decay"],
                                                    momentum=HYPER["momentum"], grad_scale=HYPER["grad_scale"])


@pytest.mark.parametrize("kind", ["sgd", "adamw"])
@pytest.mark.parametrize("n", [1003, 4096, 5])
@pytest.mark.parametrize("pdt", ["f32", "bf16"])
def test_update_of_one_tensor_over_four_steps(kind, n, pdt):
    w0 = S.normal(41, "w", (n,)) * 0.05
    if pdt == "bf16":
        w0 = S.round_bf16(w0)
    master = dev(w0, torch.float32)
    params = master if pdt == "f32" else dev(w0, torch.bfloat16)
    pop = None if pdt == "f32" else torch.zeros(n, dtype=torch.float16, device="cuda")
    m = torch.zeros(n, dtype=torch.float32, device="cuda")
    v = torch.zeros(n, dtype=torch.float32, device="cuda")
    wr, mr, vr = w0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t in range(1, 5):
        g = S.normal(41, f"g{t}", (n,)) * (1e-2 if t % 2 else 3.0)
        Bd.lsk_optimizer(0 if kind == "sgd" else 1, dev(g, torch.float32), m, v if kind == "adamw" else None,
                         master, params, pop, step=t, **HYPER)
        wr, mr, vr = O.optimizer_step(kind, wr, g.astype(np.float32), mr, vr, t, **oracle_kwargs(kind))
    assert_close(host(master), wr, 1e-5, "master weights")
    assert_close(host(m), mr, 1e-5, "first moment / momentum")
    if kind == "adamw":
        assert_close(host(v), vr, 1e-5, "second moment")
    if pdt == "bf16":
        assert torch.equal(params, master.to(torch.bfloat16))            # stored parameter = round(master)
        assert torch.equal(pop, params.to(torch.float32).to(torch.float16))   # operand copy = convert(stored)


def test_update_rejects_bad_arguments():
    z = torch.zeros(8, dtype=torch.float32, device="cuda")
    with pytest.raises(Bd.LsError):
        Bd.lsk_optimizer(2, z, z, z, z, z, None, lr=1e-3, step=1)
    with pytest.raises(Bd.LsError):
        Bd.lsk_optimizer(1, z, z, z, z, z, None, lr=1e-3, step=0)
    with pytest.raises(Bd.LsError):
        Bd.lsk_optimizer(1, z, z, None, z, z, None, lr=1e-3, step=1)


@pytest.mark.parametrize("which,kind", [("llama", "adamw"), ("gpt", "sgd")])
def test_stage_update_then_serving_uses_the_new_weights(which, kind):
    """train fwd+bwd -> update -> prefill: the update matches the oracle's rule applied to the GPU's
    own gradients (decay on weight matrices only), and the prefill that follows on the same
    stream is the oracle's forward with the updated, re-rounded weights."""
    cfg = SMALL_GPT if which == "gpt" else SMALL_LLAMA
    st, flat, pd = make_stage(cfg, mma="f16", io="f32")
    n, d = flat.size, cfg["d_model"]
    B, L = 2, 48
    X = S.make_activations(cfg, "X", (B, L, d))
    dY = S.make_activations(cfg, "dY", (B, L, d))
    ws, saved = st.new_workspace(B * L), st.new_saved(B, L)
    Y = torch.empty(B, L, d, dtype=st.io_torch, device="cuda")
    dX = torch.empty_like(Y)
    dP = torch.empty(n, dtype=torch.float32, device="cuda")
    st.stage_train_fwd(dev(X, st.io_torch), B, L, Y, saved, ws)
    st.stage_train_bwd(dev(dY, st.io_torch), B, L, saved, dX, dP, 0, ws)
    master = dev(flat, torch.float32)
    m = torch.zeros(n, dtype=torch.float32, device="cuda")
    v = torch.zeros(n, dtype=torch.float32, device="cuda")
    big = dict(HYPER, lr=2e-2)     # large enough to move every bf16 weight
    st.stage_optimizer_step(pd, master, m, v if kind == "adamw" else None, dP,
                            kind=Bd.LS_OPT_ADAMW if kind == "adamw" else Bd.LS_OPT_SGD, step=1, **big)
    # serving call enqueued right after the update, no synchronisation in between
    Xs = S.make_activations(cfg, "Xs", (40, d))
    ctx0 = np.zeros(1, np.int64)
    table, n_pages = S.page_tables(ctx0, np.array([40]), cfg["page_size"])
    kv = Bd.KV(st, n_pages, table, ctx0)
    Ys = torch.empty(40, d, dtype=st.io_torch, device="cuda")
    st.stage_prefill(dev(Xs, st.io_torch), [40], kv, Ys, st.new_workspace(40))
    torch.cuda.synchronize()
    ok = oracle_kwargs(kind)
    ok["lr"] = 2e-2
    wr, mr, vr = O.optimizer_step(kind, flat, host(dP), np.zeros(n), np.zeros(n), 1, decay=O.decay_mask(cfg), **ok)
    assert_close(host(master), wr, 1e-5, "stage master weights")
    assert_close(host(m), mr, 1e-5, "stage first moment")
    assert torch.equal(pd, master.to(torch.bfloat16))
    assert float((host(pd) != flat).mean()) > 0.5, "the update must have moved the stored weights"
    # forward with the weights the stage now holds
    cache = O.new_cache(cfg, 1)
    ys = O.stage_prefill(cfg, host(pd), [Xs.astype(np.float64)], cache)
    assert_close(host(Ys), ys[0], TOL["bf16"], "prefill after the update")
    # and it differs from the forward with the old weights by more than the tolerance
    ys_old = O.stage_prefill(cfg, flat.astype(np.float64), [Xs.astype(np.float64)], O.new_cache(cfg, 1))
    assert np.abs(ys_old[0] - ys[0]).max() > 4 * TOL["bf16"] * np.sqrt((ys[0] ** 2).mean())
    st.close()


def test_offline_profiler_sweep_runs_the_stage_and_reduces_its_timings():
    """Small stage, tiny sweep: every timing is positive, backward costs more than forward, the
    memory demand grows with C * l, and the summary carries the paper's coefficients."""
    from paper_2507_21276_amd import profiler as PR
    rows = PR.sweep(SMALL_LLAMA, [1, 2], [64, 128], reps=2)
    assert len(rows) == 4
    for r in rows:
        assert r["train_fwd_s"] > 0 and r["train_bwd_s"] > r["train_fwd_s"] * 0.8 and r["prefill_s"] > 0
    assert rows[-1]["saved_bytes"] > rows[0]["saved_bytes"]
    s = PR.summarise(rows, kappa=0.9)
    # the library's reduction of the samples it measured itself, against the oracle's plain loops
    from oracle import profile_oracle as PO
    for key, name in (("train_fwd_s", "eta_F_train"), ("prefill_s", "eta_F_prefill"), ("train_bwd_s", "eta_B")):
        samples = [(r["C"], r["l"], r[key]) for r in rows]
        assert s[name]["eta_s_per_token_sq"] == pytest.approx(PO.eta(samples), rel=1e-12)
        assert s[name]["worst_rel_err"] == pytest.approx(PO.worst_relative_error(PO.eta(samples), samples), rel=1e-9)
    demand = [r["saved_bytes"] + r["workspace_bytes"] for r in rows]
    assert s["M_peak_bytes"] == max(demand)
    assert s["M_threshold_bytes"] == pytest.approx(PO.memory_threshold(0.9, demand), rel=1e-15)
