// Offline profiler of one stage (Offline Profiling): timing of the stage calls between HIP events and the
// reduction of the samples to eta = mean(t / (C l^2)), its prediction error, two least-squares refinements,
// and M_threshold = kappa * M_peak.
#include <cmath>
#include <set>
#include <utility>
#include <vector>

#include "../../include/lemix_profile.h"
#include "common.h"

namespace {

struct EventPair {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  ~EventPair() {
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  }
};

// seconds per call of `fn`, after one untimed call
template <class F>
ls_status time_calls(F fn, hipStream_t st, int reps, double* seconds) {
  EventPair ev;
  LS_CHECK_HIP(hipEventCreate(&ev.e0));
  LS_CHECK_HIP(hipEventCreate(&ev.e1));
  LS_TRY(fn());
  LS_CHECK_HIP(hipStreamSynchronize(st));
  LS_CHECK_HIP(hipEventRecord(ev.e0, st));
  for (int i = 0; i < reps; ++i) LS_TRY(fn());
  LS_CHECK_HIP(hipEventRecord(ev.e1, st));
  LS_CHECK_HIP(hipEventSynchronize(ev.e1));
  float ms = 0.f;
  LS_CHECK_HIP(hipEventElapsedTime(&ms, ev.e0, ev.e1));
  *seconds = (double)ms * 1e-3 / reps;
  return LS_OK;
}

// Gauss-Jordan with partial pivoting on the n x n normal equations held in A[n][n + 1]
bool solve(double A[3][4], int n) {
  for (int i = 0; i < n; ++i) {
    int piv = i;
    for (int r = i + 1; r < n; ++r)
      if (std::fabs(A[r][i]) > std::fabs(A[piv][i])) piv = r;
    if (std::fabs(A[piv][i]) < 1e-300) return false;
    for (int c = 0; c <= n; ++c) std::swap(A[i][c], A[piv][c]);
    for (int r = 0; r < n; ++r) {
      if (r == i) continue;
      const double f = A[r][i] / A[i][i];
      for (int c = i; c <= n; ++c) A[r][c] -= f * A[i][c];
    }
  }
  for (int i = 0; i < n; ++i) A[i][n] /= A[i][i];
  return true;
}

}  // namespace

extern "C" {

ls_status ls_profile_reduce(const ls_profile_sample* s, int n, ls_profile_fit* out) {
  LS_REQUIRE(s && out && n >= 1, "profile_reduce: no samples");
  for (int i = 0; i < n; ++i)
    LS_REQUIRE(s[i].C >= 1 && s[i].l >= 1 && s[i].seconds > 0.0, "profile_reduce: sample %d is (C=%d, l=%d, %g s)", i,
               s[i].C, s[i].l, s[i].seconds);
  ls_profile_fit f{};
  const double nan = std::nan("");
  f.a2 = f.b2 = f.two_term_worst_rel_err = f.c3 = f.a3 = f.b3 = f.three_term_worst_rel_err = nan;
  // eta: the average of the normalised times (not a least-squares fit: every sample weighs the same)
  double sum = 0.0;
  for (int i = 0; i < n; ++i) sum += s[i].seconds / ((double)s[i].C * s[i].l * s[i].l);
  f.eta = sum / n;
  double worst = 0.0, mean = 0.0;
  for (int i = 0; i < n; ++i) {
    const double e = std::fabs(f.eta * s[i].C * (double)s[i].l * s[i].l - s[i].seconds) / s[i].seconds;
    worst = e > worst ? e : worst;
    mean += e;
  }
  f.worst_rel_err = worst;
  f.mean_rel_err = mean / n;
  std::set<int> ls_, cls;
  std::set<std::pair<int, int>> shapes;
  for (int i = 0; i < n; ++i) {
    ls_.insert(s[i].l);
    cls.insert(s[i].C * s[i].l);
    shapes.insert({s[i].C, s[i].l});
  }
  // least squares for t = sum_r coef[r] x_r with x = (C l, C l^2) or (1, C l, C l^2)
  auto fit = [&](int terms, double* coef, double* worst_out) {
    auto basis = [&](int i, double* x) {
      const double cl = (double)s[i].C * s[i].l;
      int k = 0;
      if (terms == 3) x[k++] = 1.0;
      x[k++] = cl;
      x[k++] = cl * s[i].l;
    };
    double M[3][4] = {};
    for (int i = 0; i < n; ++i) {
      double x[3];
      basis(i, x);
      for (int r = 0; r < terms; ++r) {
        for (int c = 0; c < terms; ++c) M[r][c] += x[r] * x[c];
        M[r][terms] += x[r] * s[i].seconds;
      }
    }
    if (!solve(M, terms)) return false;
    double w = 0.0;
    for (int i = 0; i < n; ++i) {
      double x[3], p = 0.0;
      basis(i, x);
      for (int r = 0; r < terms; ++r) p += M[r][terms] * x[r];
      const double e = std::fabs(p - s[i].seconds) / s[i].seconds;
      w = e > w ? e : w;
    }
    for (int r = 0; r < terms; ++r) coef[r] = M[r][terms];
    *worst_out = w;
    return true;
  };
  if (ls_.size() >= 2) {
    double c[3];
    if (fit(2, c, &f.two_term_worst_rel_err)) {
      f.a2 = c[0];
      f.b2 = c[1];
      f.has_two_term = 1;
    } else {
      f.two_term_worst_rel_err = nan;
    }
  }
  if (cls.size() >= 3 && shapes.size() >= 4) {
    double c[3];
    if (fit(3, c, &f.three_term_worst_rel_err)) {
      f.c3 = c[0];
      f.a3 = c[1];
      f.b3 = c[2];
      f.has_three_term = 1;
    } else {
      f.three_term_worst_rel_err = nan;
    }
  }
  *out = f;
  return LS_OK;
}

ls_status ls_profile_memory_threshold(double kappa, const double* demand, int n, double* m_peak, double* m_threshold) {
  LS_REQUIRE(demand && n >= 1 && m_peak && m_threshold, "profile_memory_threshold: no samples");
  LS_REQUIRE(kappa > 0.0 && kappa <= 1.0, "profile_memory_threshold: kappa %g outside (0, 1]", kappa);
  double peak = demand[0];
  for (int i = 1; i < n; ++i) peak = demand[i] > peak ? demand[i] : peak;
  *m_peak = peak;
  *m_threshold = kappa * peak;
  return LS_OK;
}

ls_status ls_profile_time_train(ls_stage* s, const void* X, int B, int L, void* Y, void* saved, const void* dY, void* dX,
                                float* dParams, void* workspace, void* stream, int reps, double* fwd_seconds,
                                double* bwd_seconds) {
  LS_REQUIRE(reps >= 1 && fwd_seconds && bwd_seconds, "profile_time_train: bad reps or null result");
  hipStream_t st = (hipStream_t)stream;
  LS_TRY(time_calls([&] { return stage_train_fwd(s, X, B, L, Y, saved, workspace, stream); }, st, reps, fwd_seconds));
  return time_calls([&] { return stage_train_bwd(s, dY, B, L, saved, dX, dParams, 0, workspace, stream); }, st, reps,
                    bwd_seconds);
}

ls_status ls_profile_time_prefill(ls_stage* s, const void* X, const int32_t* chunk_len, int B, const ls_kv* kv, void* Y,
                                  void* workspace, void* stream, int reps, double* seconds) {
  LS_REQUIRE(reps >= 1 && seconds, "profile_time_prefill: bad reps or null result");
  return time_calls([&] { return stage_prefill(s, X, chunk_len, B, kv, Y, workspace, stream); }, (hipStream_t)stream, reps,
                    seconds);
}

}  // extern "C"
