"""CPU oracle for the offline profiler's coefficients.  TEST INFRASTRUCTURE.

Only tests may import this file; it shares no code with the package.

Offline Profiling (Latency estimation) models a stage's forward and backward time as
Delta = eta * C * l^2 (C = batch size, l = query length) and obtains eta by measuring stage
run times over several (C, l) and normalising each by C * l^2; the coefficient is the average
of the normalised times.  Memory profiling sets M_threshold = kappa * M_peak, M_peak being the
largest memory demand seen over the sweep.  Both are written out as plain loops.
"""


def eta(samples):
    """samples: iterable of (C, l, seconds).  Mean of seconds / (C * l^2)."""
    total, n = 0.0, 0
    for C, l, t in samples:
        total += t / (C * l * l)
        n += 1
    if n == 0:
        raise ValueError("no samples")
    return total / n


def predicted(eta_value, C, l):
    """Delta = eta * C * l^2."""
    return eta_value * C * l * l


def worst_relative_error(eta_value, samples):
    """max over samples of |eta C l^2 - t| / t."""
    worst = 0.0
    for C, l, t in samples:
        worst = max(worst, abs(predicted(eta_value, C, l) - t) / t)
    return worst


def memory_threshold(kappa, demands):
    """kappa * max(demands)."""
    peak = None
    for m in demands:
        peak = m if peak is None or m > peak else peak
    if peak is None:
        raise ValueError("no samples")
    return kappa * peak
