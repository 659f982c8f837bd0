"""Offline profiler: the oracle's pins and the library's reduction (include/lemix_profile.h, host code) against
the oracle (CPU only)."""
import math

import pytest

from oracle import profile_oracle as PO
from paper_2507_21276_amd import profiler as PR


def make(eta, shapes, noise=None):
    return [(C, l, eta * C * l * l * (1.0 if noise is None else noise[i])) for i, (C, l) in enumerate(shapes)]


SHAPES = [(1, 128), (2, 128), (1, 512), (4, 1024), (2, 2048)]


def test_oracle_recovers_an_exact_quadratic_law():
    s = make(3.5e-9, SHAPES)
    assert PO.eta(s) == pytest.approx(3.5e-9, rel=1e-14)
    assert PO.worst_relative_error(3.5e-9, s) < 1e-14


def test_oracle_eta_is_the_mean_of_the_normalised_times_not_a_least_squares_fit():
    # two samples whose normalised times are 1 and 3: the paper's average is 2 whatever their sizes
    s = [(1, 10, 1.0 * 100), (1, 1000, 3.0 * 1e6)]
    assert PO.eta(s) == pytest.approx(2.0)
    # a least-squares fit would be pulled to ~3 by the large sample
    ls = sum(t * C * l * l for C, l, t in s) / sum((C * l * l) ** 2 for C, l, t in s)
    assert ls > 2.9


def test_oracle_eta_is_linear_in_the_times_and_batch_invariant_under_the_law():
    s = make(2e-9, SHAPES, noise=[1.1, 0.9, 1.0, 1.2, 0.8])
    assert PO.eta([(C, l, 3 * t) for C, l, t in s]) == pytest.approx(3 * PO.eta(s))
    assert PO.eta([(2 * C, l, 2 * t) for C, l, t in s]) == pytest.approx(PO.eta(s))


def test_oracle_memory_threshold():
    assert PO.memory_threshold(0.9, [3.0, 10.0, 7.0]) == pytest.approx(9.0)
    with pytest.raises(ValueError):
        PO.memory_threshold(0.9, [])
    with pytest.raises(ValueError):
        PO.eta([])


def test_library_reduction_matches_the_oracle():
    s = make(7e-10, SHAPES, noise=[1.3, 0.7, 1.0, 1.05, 0.95])
    f = PR.ls_profile_reduce(s)
    assert f["eta"] == pytest.approx(PO.eta(s), rel=1e-14)
    assert f["worst_rel_err"] == pytest.approx(PO.worst_relative_error(PO.eta(s), s), rel=1e-12)
    mean = sum(abs(PO.predicted(PO.eta(s), C, l) - t) / t for C, l, t in s) / len(s)
    assert f["mean_rel_err"] == pytest.approx(mean, rel=1e-12)
    assert PR.ls_profile_memory_threshold(0.8, [1e9, 5e9]) == (5e9, PO.memory_threshold(0.8, [1e9, 5e9]))
    # the average of the normalised times, not a least-squares fit (the oracle's own pin, through the library)
    assert PR.ls_profile_reduce([(1, 10, 1.0 * 100), (1, 1000, 3.0 * 1e6)])["eta"] == pytest.approx(2.0)
    from paper_2507_21276_amd import binding as Bd
    for bad in ([], [(0, 10, 1.0)], [(1, 10, 0.0)], [(1, 0, 1.0)]):
        with pytest.raises(Bd.LsError):
            PR.ls_profile_reduce(bad)
    for kappa, demands in ((0.9, []), (0.0, [1.0]), (1.5, [1.0])):
        with pytest.raises(Bd.LsError):
            PR.ls_profile_memory_threshold(kappa, demands)


def test_two_term_fit_recovers_linear_and_quadratic_parts():
    a, b = 4e-7, 2e-10
    s = [(C, l, a * C * l + b * C * l * l) for C, l in SHAPES]
    f = PR.ls_profile_reduce(s)
    assert f["has_two_term"] == 1 and f["a2"] == pytest.approx(a, rel=1e-9) and f["b2"] == pytest.approx(b, rel=1e-9)
    assert f["two_term_worst_rel_err"] < 1e-9
    one = PR.ls_profile_reduce([(1, 100, 1.0)])     # one length cannot separate l from l^2
    assert one["has_two_term"] == 0 and math.isnan(one["a2"])


def test_summary_shape():
    rows = [{"C": C, "l": l, "train_fwd_s": 1e-9 * C * l * l, "train_bwd_s": 2e-9 * C * l * l,
             "prefill_s": float("nan") if C > 2 else 1.1e-9 * C * l * l, "saved_bytes": 1000 * C * l,
             "workspace_bytes": 10 * C * l} for C, l in SHAPES]
    out = PR.summarise(rows, kappa=0.5)
    assert out["eta_F_train"]["eta_s_per_token_sq"] == pytest.approx(1e-9)
    assert out["eta_B"]["eta_s_per_token_sq"] == pytest.approx(2e-9)
    assert out["eta_F_prefill"]["worst_rel_err"] < 1e-12
    assert out["M_peak_bytes"] == 1010 * 2 * 2048 and out["M_threshold_bytes"] == 0.5 * 1010 * 2 * 2048
    assert not math.isnan(out["eta_B"]["b_s_per_token_sq"])


def test_three_term_fit_recovers_a_floor():
    c0, a, b = 2e-3, 4e-7, 2e-10
    shapes = SHAPES + [(4, 256), (1, 2048)]
    s = [(C, l, c0 + a * C * l + b * C * l * l) for C, l in shapes]
    f = PR.ls_profile_reduce(s)
    assert f["has_three_term"] == 1 and f["three_term_worst_rel_err"] < 1e-6
    assert f["c3"] == pytest.approx(c0, rel=1e-6) and f["a3"] == pytest.approx(a, rel=1e-6) and f["b3"] == pytest.approx(b, rel=1e-6)
    assert PR.ls_profile_reduce([(1, 100, 1.0), (2, 100, 2.0)])["has_three_term"] == 0
