"""Offline profiler of one stage (Offline Profiling: latency and memory coefficients).

Sweeps batch size C and query length l, times the stage's forward (prefill and training
forward) and backward with HIP events, and reduces the timings the way the paper does:
eta = mean of time / (C l^2) for forward and for backward, M_threshold = kappa * M_peak with
the stage's own memory demand (saved activations + workspace) as the profile.  It also reports
how well eta C l^2 predicts each sample, and the coefficients of the two-term form
a C l + b C l^2, which separates the linear (projection / FFN) from the quadratic (attention)
part of a decoder block.  Every timed step runs in the HIP kernels through the C ABI; this
module only marshals arguments and averages numbers.

    python -m paper_2507_21276_amd.profiler --stage llama7b_bf16 --C 1 2 4 --L 256 512 1024 2048
"""
from __future__ import annotations

import argparse
import json
import sys
from typing import Iterable, List, Sequence, Tuple

Sample = Tuple[int, int, float]   # (C, l, seconds)


def fit_eta(samples: Iterable[Sample]) -> float:
    """The paper's coefficient: average of the run times normalised by C l^2."""
    vals = [t / (C * l * l) for C, l, t in samples]
    if not vals:
        raise ValueError("fit_eta: no samples")
    return sum(vals) / len(vals)


def relative_errors(eta: float, samples: Iterable[Sample]) -> List[float]:
    return [abs(eta * C * l * l - t) / t for C, l, t in samples]


def fit_linear_quadratic(samples: Sequence[Sample]) -> Tuple[float, float]:
    """Least squares for t = a C l + b C l^2 (normal equations of the 2-column problem)."""
    s11 = s12 = s22 = r1 = r2 = 0.0
    for C, l, t in samples:
        x1, x2 = C * l, C * l * l
        s11 += x1 * x1
        s12 += x1 * x2
        s22 += x2 * x2
        r1 += x1 * t
        r2 += x2 * t
    det = s11 * s22 - s12 * s12
    if det == 0.0:
        raise ValueError("fit_linear_quadratic: the samples do not separate l from l^2")
    return (r1 * s22 - r2 * s12) / det, (r2 * s11 - r1 * s12) / det


def fit_floor_linear_quadratic(samples: Sequence[Sample]) -> Tuple[float, float, float]:
    """Least squares for t = c0 + a C l + b C l^2: c0 is the floor of a call that mostly streams
    the stage's weights (small batches), which neither of the other two forms can express."""
    A = [[0.0] * 4 for _ in range(3)]
    for C, l, t in samples:
        x = (1.0, float(C * l), float(C * l * l))
        for i in range(3):
            for j in range(3):
                A[i][j] += x[i] * x[j]
            A[i][3] += x[i] * t
    for i in range(3):   # Gauss-Jordan with partial pivoting on the 3 x 3 normal equations
        piv = max(range(i, 3), key=lambda r: abs(A[r][i]))
        if abs(A[piv][i]) < 1e-300:
            raise ValueError("fit_floor_linear_quadratic: the samples do not determine three coefficients")
        A[i], A[piv] = A[piv], A[i]
        for r in range(3):
            if r != i:
                f = A[r][i] / A[i][i]
                for c in range(i, 4):
                    A[r][c] -= f * A[i][c]
    return A[0][3] / A[0][0], A[1][3] / A[1][1], A[2][3] / A[2][2]


def memory_threshold(kappa: float, demands: Iterable[float]) -> float:
    demands = list(demands)
    if not demands:
        raise ValueError("memory_threshold: no samples")
    return kappa * max(demands)


def sweep(cfg: dict, Cs: Sequence[int], Ls: Sequence[int], reps: int = 3, mma: str = "f16", io: str = "bf16"):
    """Times stage_train_fwd, stage_train_bwd and stage_prefill for every (C, l).  Returns a list
    of dicts with seconds per call and the stage's memory demand in bytes."""
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

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    for C in Cs:
        for L in Ls:
            T = C * L
            X = S.normal_torch(0, "X", (C, L, d), 1.0, "cuda", st.io_torch)
            dY = S.normal_torch(0, "dY", (C, L, d), 1.0, "cuda", st.io_torch)
            Y, dX = torch.empty_like(X), torch.empty_like(X)
            ws, saved = st.new_workspace(T), st.new_saved(C, L)
            t_f = timed(lambda: st.stage_train_fwd(X, C, L, Y, saved, ws))
            t_b = timed(lambda: st.stage_train_bwd(dY, C, L, saved, dX, dP, 0, ws))
            ctx0 = np.zeros(C, np.int64)
            table, n_pages = S.page_tables(ctx0, np.full(C, L), P)
            kv = Bd.KV(st, n_pages, table, ctx0)
            Xp, Yp = X.reshape(T, d), Y.reshape(T, d)
            t_p = timed(lambda: st.stage_prefill(Xp, [L] * C, kv, Yp, ws)) if C <= 32 else float("nan")
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
        eta = fit_eta(samples)
        errs = relative_errors(eta, samples)
        a, b = fit_linear_quadratic(samples) if len({(C, l) for C, l, _ in samples}) > 1 else (float("nan"),) * 2
        errs2 = [abs(a * C * l + b * C * l * l - t) / t for C, l, t in samples] if a == a else []
        out[name] = {"eta_s_per_token_sq": eta, "worst_rel_err": max(errs), "mean_rel_err": sum(errs) / len(errs),
                     "a_s_per_token": a, "b_s_per_token_sq": b,
                     "two_term_worst_rel_err": max(errs2) if errs2 else float("nan")}
        if len({C * l for C, l, _ in samples}) >= 3 and len({(C, l) for C, l, _ in samples}) >= 4:
            c0, a3, b3 = fit_floor_linear_quadratic(samples)
            errs3 = [abs(c0 + a3 * C * l + b3 * C * l * l - t) / t for C, l, t in samples]
            out[name].update({"floor_s": c0, "floor_a_s_per_token": a3, "floor_b_s_per_token_sq": b3,
                              "three_term_worst_rel_err": max(errs3)})
    demand = [r["saved_bytes"] + r["workspace_bytes"] for r in rows]
    out["M_peak_bytes"] = max(demand)
    out["M_threshold_bytes"] = memory_threshold(kappa, demand)
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
