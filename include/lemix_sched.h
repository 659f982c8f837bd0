/*
 * lemix_sched.h - C ABI of the host-side scheduling steps that drive the stage.
 *
 * Everything here is host bookkeeping: no argument is device memory and no
 * call touches the GPU.  The steps are the paper's own:
 *   - Task-Specific Execution Planning, Algorithm 1 (ComputeIdleness) and the
 *     "Backward planning" paragraph: ls_node_plan;
 *   - Hierarchical Resource Allocation, Eq. 1 (idleness profit), Eq. 2 (length
 *     consistency), Eq. 3 (node priority score): ls_node_score, ls_select_node;
 *     Eq. 4 (deprioritising a training task whose successor inference task
 *     would miss the response goal): ls_deprioritize;
 *   - Runtime Memory-Aware Scheduling, Algorithm 2 (ExecuteTaskMemoryAware):
 *     ls_node_execute, with the stage calls supplied as hooks;
 *   - Autoregressive Generation, Algorithm 3 (ContinuousBatching): ls_batcher_*.
 *
 * Conventions: times are seconds in double precision on any common clock;
 * stages are numbered 0 .. S-1 (the paper's 1 .. S); every pointer is host
 * memory owned by the caller; objects are not thread-safe (one owner thread
 * each); every call returns an ls_status and ls_last_error() describes the
 * last failure.
 *
 * Where the listings leave a choice open, this is what is done:
 *   - the new task's "stage 0" forward end is its arrival time a, and on a node
 *     whose trace queue is empty the preceding task's forward end is a at
 *     every stage;
 *   - Q_temp is a copy of Q_train taken once before the stage loop; a training
 *     task that postpones the forward is consumed (later stages no longer see
 *     it), one the forward fits in front of returns to the head;
 *   - CheckExecuted at the first stage holds for every training task that
 *     postponed the forward there (its backward path ends at that stage before
 *     the forward starts); the task leaves Q_train only when the plan is
 *     committed, never when a node is merely evaluated;
 *   - backward path of a committed training task: at the last stage it starts
 *     at max(own forward end there, backward end there of the training task
 *     committed before it); at stage s at max(own backward end at s+1, that
 *     task's backward end at s); each lasts eta_B C l^2;
 *   - Eq. 2 uses the population standard deviation of the query lengths given
 *     to the node so far and is 0 with fewer than two of them or zero spread;
 *   - Eq. 4's inner maximum is over the tasks in the node's trace queue (their
 *     forward end at the last stage) and is a' for an empty node; a training
 *     task is deprioritised when the bound is strictly greater than tau_R;
 *   - Algorithm 3 inspects the head of the queue without removing it; a
 *     training task at the head ends the admission round and stays until
 *     ls_batcher_take_training removes it.
 */
#ifndef LEMIX_SCHED_H
#define LEMIX_SCHED_H

#include <stdint.h>

#include "lemix_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ls_node ls_node;       /* one node's trace queues (opaque) */
typedef struct ls_batcher ls_batcher; /* Algorithm 3 state (opaque) */

/* A task batch {a, l, C} (Algorithm 1, Input). */
typedef struct {
  double a;                 /* arrival (enqueue) time */
  double len;               /* query length l, tokens */
  double C;                 /* batch size */
  int32_t require_backward; /* 1: training task, 0: inference task */
} ls_task;

/* S stages; eta_f, eta_b: the offline profiler's coefficients (Offline
 * Profiling: Delta_F = eta_F C l^2, Delta_B = eta_B C l^2), both >= 0. */
ls_status ls_node_create(int S, double eta_f, double eta_b, ls_node** out);
void ls_node_destroy(ls_node* n);

/*
 * Algorithm 1 for `task` on node n.  II and R are written when non-null;
 * path, when non-null, receives 4*S doubles: start_f[S], end_f[S], start_b[S],
 * end_b[S] (the backward half is zero for an inference task or when
 * commit == 0).  commit == 0 evaluates only.  commit == 1 also enqueues the
 * task with this path (planning its backward path if it is a training task),
 * removes the training tasks CheckExecuted found finished, records len in the
 * node's length history, and writes the task's id (>= 0, unique per node) to
 * *task_id when non-null.
 * LS_EINVAL: null n or task, len or C not positive or not finite, a not finite.
 */
ls_status ls_node_plan(ls_node* n, const ls_task* task, int commit, double* II, double* R,
                       double* path, int64_t* task_id);

/* Number of tasks in the trace queue (train_only == 0) or in Q_train (1). */
int ls_node_queue_len(const ls_node* n, int train_only);

/*
 * Drops, from the old end of the trace queue, tasks that Algorithm 2 has run,
 * that are no longer in Q_train and that are neither the last task nor the
 * last training task: Algorithm 1 never looks at them again.  (Eq. 4's
 * maximum then runs over what remains; forward ends grow along the queue, so
 * its value does not change.)  Returns the number of tasks dropped.
 */
int ls_node_prune(ls_node* n);

/* The recorded path of a committed task: 4*S doubles as for ls_node_plan.
 * LS_EINVAL for an unknown id. */
ls_status ls_node_task_path(const ls_node* n, int64_t task_id, double* path);

/*
 * Calibration (Algorithm 2, "Calibrate"): replace the planned interval of a
 * committed task at one stage by the measured one.  backward == 0: forward
 * interval, 1: backward interval.  LS_EINVAL for an unknown id or stage.
 */
ls_status ls_node_calibrate(ls_node* n, int64_t task_id, int stage, int backward, double start,
                            double end);

/* Eq. 1-3 parameters. */
typedef struct {
  double tau;     /* threshold of Eq. 1 */
  double lambda1; /* weight of the response time R in Eq. 3, > 0 */
  double lambda2; /* weight of the length consistency LC in Eq. 3 */
} ls_score_params;

/*
 * Priority score of node n for `task` (Eq. 3), from Algorithm 1's II and R,
 * IP = -max(II / S - (a - a_prev), tau) (Eq. 1; a_prev is the arrival time of
 * the task before this one) and LC (Eq. 2).  Outputs may be null.  Changes
 * nothing in n.
 */
ls_status ls_node_score(ls_node* n, const ls_task* task, double a_prev, const ls_score_params* p,
                        double* f, double* IP, double* LC, double* II, double* R);

/* Index of the node with the highest score among nodes[0..N-1] (the first of
 * equal scores); scores, when non-null, receives the N values. */
ls_status ls_select_node(ls_node* const* nodes, int N, const ls_task* task, double a_prev,
                         const ls_score_params* p, int* best, double* scores);

/*
 * Eq. 4 for the inference task `next` that follows a training task in the
 * global queue: bound = min over nodes of (latest forward end at the last
 * stage among the node's queued tasks + eta_F^n C' l'^2) - a'.
 * *deprioritize = 1 when bound > tau_R.  Outputs may be null.
 */
ls_status ls_deprioritize(ls_node* const* nodes, int N, const ls_task* next, double tau_R,
                          int* deprioritize, double* bound);

/*
 * Algorithm 2.  The stage work and the memory test are the caller's: on the
 * GPU they are stage_* calls, lsk_memory_available and lsk_kv_offload; a test
 * supplies scripted ones.  All hooks are required.
 */
typedef struct {
  void* ctx;
  int (*memory_available)(void* ctx, int stage);                 /* MemoryAvailable(n, s, M_threshold) */
  void (*wait)(void* ctx, double seconds);                       /* lets the check interval pass */
  void (*offload)(void* ctx, int64_t task_id, int stage);        /* offload the task's KV cache from stage s */
  void (*forward)(void* ctx, int64_t task_id, int stage, double* start, double* end);
  void (*backward)(void* ctx, int64_t task_id, double* start, double* end); /* S entries each */
} ls_exec_hooks;

typedef struct {
  int64_t tasks, forwards, backwards, offloads, skipped_forwards;
  double waited; /* sum of check intervals spent waiting */
} ls_exec_stats;

/*
 * Runs every committed, not yet executed task of node n in queue order: per
 * stage, waits in steps of dt while memory is unavailable; once the wait
 * reaches t_max it offloads the task's KV cache from that stage and stops
 * waiting; runs the forward if memory is then available (otherwise that
 * stage's forward is skipped, as in the listing) and calibrates the recorded
 * interval; after the last stage of a training task runs the backward and
 * calibrates its intervals.  dt > 0, t_max >= 0.  stats may be null.
 */
ls_status ls_node_execute(ls_node* n, double dt, double t_max, const ls_exec_hooks* hooks,
                          ls_exec_stats* stats);

/* Algorithm 3.  C >= 1: maximum batch size; T_w >= 0: maximum waiting time. */
ls_status ls_batcher_create(int C, double T_w, ls_batcher** out);
void ls_batcher_destroy(ls_batcher* b);

/* Appends a request to the node's task queue (FCFS order). */
ls_status ls_batcher_push(ls_batcher* b, int64_t request_id, int require_backward);

/*
 * One pass of the loop body up to "Execute batch": if the batch is empty the
 * batch start time becomes `now`; then requests join from the head of the
 * queue while the batch holds fewer than C, the head is an inference request
 * and batch start + T_w > now.  batch_ids (capacity C) receives the whole
 * batch, continuing requests first in their order of admission, then the
 * *n_new requests admitted by this call.  *head_is_training = 1 when a
 * training task at the head stopped the admission.
 */
ls_status ls_batcher_form(ls_batcher* b, double now, int64_t* batch_ids, int* n_batch, int* n_new,
                          int* head_is_training);

/* Removes the training task at the head of the queue; *request_id = -1 and
 * LS_OK when the head is not a training task. */
ls_status ls_batcher_take_training(ls_batcher* b, int64_t* request_id);

/* filter_finished_requests: drops the listed ids from the batch. */
ls_status ls_batcher_finish(ls_batcher* b, const int64_t* finished_ids, int n);

/* Requests waiting in the queue / held in the batch. */
int ls_batcher_queued(const ls_batcher* b);
int ls_batcher_batch_size(const ls_batcher* b);

#ifdef __cplusplus
}
#endif
#endif /* LEMIX_SCHED_H */
