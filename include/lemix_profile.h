/*
 * lemix_profile.h - the offline profiler of one stage (Offline Profiling:
 * latency estimation and memory profiling).
 *
 * The paper models a stage's forward and backward time on a task batch
 * {l, C} as Delta = eta * C * l^2, obtains eta_F and eta_B by timing the stage
 * over several (C, l) and averaging the times normalised by C * l^2, and sets
 * the memory threshold of Algorithm 2 to M_threshold = kappa * M_peak, M_peak
 * being the largest demand seen.  Both steps live here: the two timing calls
 * run the stage's own entry points between HIP events, and the reduction turns
 * samples into eta, the quality of eta * C * l^2 as a predictor, and - because
 * at short l a decoder block's time is dominated by its projections, which are
 * linear in l - the least-squares coefficients of a C l + b C l^2 and of
 * c + a C l + b C l^2.
 *
 * Pointers marked [dev] are device memory owned by the caller, everything else
 * is host memory; statuses and ls_last_error() as in lemix_stage.h.
 */
#ifndef LEMIX_PROFILE_H
#define LEMIX_PROFILE_H

#include "lemix_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

/* One timed stage call on a batch of C sequences of l tokens. */
typedef struct {
  int32_t C, l;
  double seconds;
} ls_profile_sample;

typedef struct {
  /* the paper's coefficient: mean over the samples of seconds / (C l^2), and how well
   * eta C l^2 reproduces each sample: |eta C l^2 - t| / t, worst and mean */
  double eta, worst_rel_err, mean_rel_err;
  /* t = a C l + b C l^2 (needs two different l; has_two_term = 0 and NaNs otherwise) */
  double a2, b2, two_term_worst_rel_err;
  /* t = c + a C l + b C l^2 (needs three different C l and four different (C, l)) */
  double c3, a3, b3, three_term_worst_rel_err;
  int32_t has_two_term, has_three_term;
} ls_profile_fit;

/* Reduces n >= 1 samples (C, l >= 1, seconds > 0).  LS_EINVAL otherwise. */
ls_status ls_profile_reduce(const ls_profile_sample* samples, int n, ls_profile_fit* out);

/* M_peak = max of the n >= 1 demands (bytes), M_threshold = kappa * M_peak, 0 < kappa <= 1. */
ls_status ls_profile_memory_threshold(double kappa, const double* demand_bytes, int n, double* m_peak,
                                      double* m_threshold);

/*
 * Times stage_train_fwd and stage_train_bwd on one micro-batch: one untimed
 * call of each, then `reps` calls of the forward between two HIP events on
 * `stream`, then `reps` calls of the backward likewise; writes seconds per
 * call.  Arguments as the two stage calls ([dev] buffers, accumulate = 0).
 * Synchronises the stream.
 */
ls_status ls_profile_time_train(ls_stage* s, const void* X, int B, int L, void* Y, void* saved, const void* dY,
                                void* dX, float* dParams, void* workspace, void* stream, int reps,
                                double* fwd_seconds, double* bwd_seconds);

/* The same for stage_prefill (arguments as that call; the K/V rows land at the
 * same positions every repetition since ctx_len is not advanced). */
ls_status ls_profile_time_prefill(ls_stage* s, const void* X, const int32_t* chunk_len, int B, const ls_kv* kv,
                                  void* Y, void* workspace, void* stream, int reps, double* seconds);

#ifdef __cplusplus
}
#endif
#endif /* LEMIX_PROFILE_H */
