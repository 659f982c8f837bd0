"""Offline profiler of one stage (Offline Profiling: latency and memory coefficients).

Sweeps batch size C and query length l, times the stage's forward (prefill and training
forward) and backward with HIP events, and reduces the timings the way the paper does:
eta = mean of time / (C l^2) for forward and for backward, M_threshold = kappa * M_peak with
the stage's own memory demand (saved activations + workspace) as the profile.  Timing (HIP
events around the stage calls) and reduction (eta, how well eta C l^2 predicts each sample,
the coefficients of a C l + b C l^2 and c + a C l + b C l^2) both happen inside the library
(include/lemix_profile.h); this module allocates the tensors of the sweep and marshals.

    python -m paper_2507_21276_amd.profiler --stage llama7b_bf16 --C 1 2 4 --L 256 512 1024 2048
"""
from __future__ import annotations

import argparse
import json
import sys
from typing import Iterable, List, Sequence, Tuple

import ctypes as C

Sample = Tuple[int, int, float]   # (C, l, seconds)


class ls_profile_sample(C.Structure):
    _fields_ = [("C", C.c_int32), ("l", C.c_int32), ("seconds", C.c_double)]


class ls_profile_fit(C.Structure):
    _fields_ = [(k, C.c_double) for k in ("eta", "worst_rel_err", "mean_rel_err", "a2", "b2", "two_term_worst_rel_err",
                                          "c3", "a3", "b3", "three_term_worst_rel_err")] + \
               [("has_two_term", C.c_int32), ("has_three_term", C.c_int32)]


def _lib():
    from . import binding as Bd
    return Bd.lib()


def ls_profile_reduce(samples: Iterable[Sample]) -> dict:
    """The library's reduction of (C, l, seconds) samples; see include/lemix_profile.h."""
    from . import binding as Bd
    samples = list(samples)
    arr = (ls_profile_sample * max(1, len(samples)))(*[ls_profile_sample(int(c), int(l), float(t)) for c, l, t in samples])
    out = ls_profile_fit()
    Bd._check(_lib().ls_profile_reduce(arr, len(samples), C.byref(out)))
    return {k: getattr(out, k) for k, _ in ls_profile_fit._fields_}


def ls_profile_memory_threshold(kappa: float, demands: Iterable[float]) -> Tuple[float, float]:
    from . import binding as Bd
    demands = [float(v) for v in demands]
    arr = (C.c_double * max(1, len(demands)))(*demands)
    peak, thr = C.c_double(0.0), C.c_double(0.0)
    Bd._check(_lib().ls_profile_memory_threshold(kappa, arr, len(demands), C.byref(peak), C.byref(thr)))
    return peak.value, thr.value


def sweep(cfg: dict, Cs: Sequence[int], Ls: Sequence[int], reps: int = 3, mma: str = "f16", io: str = "bf16"):
    """Times stage_train_fwd, stage_train_bwd and stage_prefill for every (C, l).  Returns a list
    of dicts with seconds per call and the stage's memory demand in bytes."""
    import ctypes as Cc   # (C is the batch size in this function)
    import numpy as np
    import torch
    from . import binding as Bd
    from . import synth_inputs as S

    st = Bd.Stage(cfg, io_dtype=io if cfg["dtype"] != "f32" else None, mma_dtype=mma if cfg["dtype"] != "f32" else None)
    params = S.make_params_torch(cfg, seed=0)
    st.ls_bind_params(params)
    d, P = cfg["d_model"], cfg["page_size"]
    dP = torch.zeros(st.ls_param_count(), dtype=torch.float32, device="cuda")
    rows = []

    for C in Cs:
        for L in Ls:
            T = C * L
            X = S.normal_torch(0, "X", (C, L, d), 1.0, "cuda", st.io_torch)
            dY = S.normal_torch(0, "dY", (C, L, d), 1.0, "cuda", st.io_torch)
            Y, dX = torch.empty_like(X), torch.empty_like(X)
            ws, saved = st.new_workspace(T), st.new_saved(C, L)
            tf, tb = Cc.c_double(0.0), Cc.c_double(0.0)
            stream = Bd._stream(None)
            Bd._check(_lib().ls_profile_time_train(st.h, X.data_ptr(), C, L, Y.data_ptr(), saved.data_ptr(), dY.data_ptr(),
                                                   dX.data_ptr(), dP.data_ptr(), ws.data_ptr(), stream, reps,
                                                   Cc.byref(tf), Cc.byref(tb)))
            t_f, t_b = tf.value, tb.value
            ctx0 = np.zeros(C, np.int64)
            table, n_pages = S.page_tables(ctx0, np.full(C, L), P)
            kv = Bd.KV(st, n_pages, table, ctx0)
            Xp, Yp = X.reshape(T, d), Y.reshape(T, d)
            t_p = float("nan")
            if C <= 32:
                tp, d_ = Cc.c_double(0.0), kv.desc(True)
                Bd._check(_lib().ls_profile_time_prefill(st.h, Xp.data_ptr(), (Cc.c_int32 * C)(*([L] * C)), C, Cc.byref(d_),
                                                         Yp.data_ptr(), ws.data_ptr(), stream, reps, Cc.byref(tp)))
                t_p = tp.value
            rows.append({"C": C, "l": L, "train_fwd_s": t_f, "train_bwd_s": t_b, "prefill_s": t_p,
                         "saved_bytes": st.ls_saved_bytes(C, L), "workspace_bytes": st.ls_workspace_bytes(T)})
            del X, dY, Y, dX, ws, saved, kv
    st.close()
    return rows


def summarise(rows, kappa: float = 0.9) -> dict:
    out = {"kappa": kappa}
    for key, name in (("train_fwd_s", "eta_F_train"), ("prefill_s", "eta_F_prefill"), ("train_bwd_s", "eta_B")):
        samples = [(r["C"], r["l"], r[key]) for r in rows if r[key] == r[key]]
        if not samples:
            continue
        f = ls_profile_reduce(samples)
        out[name] = {"eta_s_per_token_sq": f["eta"], "worst_rel_err": f["worst_rel_err"], "mean_rel_err": f["mean_rel_err"],
                     "a_s_per_token": f["a2"], "b_s_per_token_sq": f["b2"],
                     "two_term_worst_rel_err": f["two_term_worst_rel_err"]}
        if f["has_three_term"]:
            out[name].update({"floor_s": f["c3"], "floor_a_s_per_token": f["a3"], "floor_b_s_per_token_sq": f["b3"],
                              "three_term_worst_rel_err": f["three_term_worst_rel_err"]})
    out["M_peak_bytes"], out["M_threshold_bytes"] = ls_profile_memory_threshold(
        kappa, [r["saved_bytes"] + r["workspace_bytes"] for r in rows])
    return out


def main(argv=None):
    from . import synth_inputs as S
    ap = argparse.ArgumentParser()
    ap.add_argument("--stage", default="llama7b_bf16", choices=sorted(S.CONFIGS))
    ap.add_argument("--C", type=int, nargs="+", default=[1, 2, 4])
    ap.add_argument("--L", type=int, nargs="+", default=[256, 512, 1024, 2048])
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--kappa", type=float, default=0.9)
    ap.add_argument("--out", default=None)
    a = ap.parse_args(argv)
    rows = sweep(S.CONFIGS[a.stage], a.C, a.L, a.reps)
    res = {"stage": a.stage, "samples": rows, "summary": summarise(rows, a.kappa)}
    text = json.dumps(res, indent=1)
    if a.out:
        with open(a.out, "w") as fh:
            fh.write(text)
    print(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
