// Host-side scheduling steps around the stage: execution planning (Algorithm 1
// and the backward-planning paragraph), node scores (Eq. 1-4), the
// memory-aware execution loop (Algorithm 2) and the continuous batcher
// (Algorithm 3).  Plain bookkeeping on the host; nothing here touches the GPU.
#include <algorithm>
#include <cmath>
#include <deque>
#include <new>
#include <vector>

#include "../../include/lemix_sched.h"
#include "common.h"

struct PlannedTask {
  int64_t id;
  double a, len, C;
  bool require_backward;
  bool in_train;   // still in Q_train
  bool executed;   // Algorithm 2 has run it
  std::vector<double> start_f, end_f, start_b, end_b;
};

struct ls_node {
  int S;
  double eta_f, eta_b;
  std::deque<PlannedTask> queue;  // Q^n in enqueue order; Q_train is the in_train subset
  int64_t next_id = 0;
  int64_t last_train = -1;        // id of the training task committed last
  // length history for Eq. 2
  std::vector<double> lens;
};

struct ls_batcher {
  int C;
  double T_w;
  struct Req { int64_t id; bool require_backward; };
  std::deque<Req> queue;
  std::vector<int64_t> batch;
  double t_start = 0;
};

namespace {

PlannedTask* find_task(ls_node* n, int64_t id) {
  for (auto& t : n->queue)
    if (t.id == id) return &t;
  return nullptr;
}
const PlannedTask* find_task(const ls_node* n, int64_t id) { return find_task(const_cast<ls_node*>(n), id); }

bool task_ok(const ls_task* t) {
  return t && std::isfinite(t->a) && std::isfinite(t->len) && std::isfinite(t->C) && t->len > 0 && t->C > 0;
}

struct Plan {
  double II, R;
  std::vector<double> start_f, end_f;
  std::vector<int64_t> removed;  // training tasks CheckExecuted found finished
};

// Algorithm 1
Plan compute_idleness(const ls_node* n, const ls_task& task) {
  const int S = n->S;
  Plan p;
  p.start_f.assign(S, 0.0);
  p.end_f.assign(S, 0.0);
  const double delta_f = n->eta_f * task.C * task.len * task.len;
  std::vector<double> prev_end(S, task.a);
  if (!n->queue.empty()) prev_end = n->queue.back().end_f;
  std::deque<const PlannedTask*> q_temp;
  for (const auto& t : n->queue)
    if (t.in_train) q_temp.push_back(&t);
  double II = 0.0, end_before = task.a;
  for (int s = 0; s < S; ++s) {
    double start = std::max(end_before, prev_end[s]);
    double end = start + delta_f;
    double offset = 0.0;
    while (!q_temp.empty()) {
      const PlannedTask* t = q_temp.front();
      if (end <= t->start_b[s]) break;  // fits in front of that backward: t stays at the head
      q_temp.pop_front();
      start = std::max(start, t->end_b[s]);
      end = start + delta_f;
      if (prev_end[s] <= t->start_b[s]) offset = offset + n->eta_b * t->C * t->len * t->len;
      if (s == 0) p.removed.push_back(t->id);
    }
    II = II + start - prev_end[s] - offset;
    p.start_f[s] = start;
    p.end_f[s] = end;
    end_before = end;
  }
  p.II = II;
  p.R = p.end_f[S - 1] - task.a;
  return p;
}

double idleness_profit(double II, int S, double a, double a_prev, double tau) {
  return -std::max(II / S - (a - a_prev), tau);
}

double length_consistency(const ls_node* n, double l) {
  const size_t cnt = n->lens.size();
  if (cnt < 2) return 0.0;
  double sum = 0.0;
  for (double x : n->lens) sum += x;
  const double mu = sum / (double)cnt;
  double var = 0.0;
  for (double x : n->lens) var += (x - mu) * (x - mu);
  var = var / (double)cnt;
  if (!(var > 0.0)) return 0.0;
  const double sigma = std::sqrt(var);
  return 1.0 / (sigma * std::sqrt(2.0 * M_PI)) * std::exp(-(l - mu) * (l - mu) / (2.0 * var));
}

void write_path(const PlannedTask& t, double* path) {
  const int S = (int)t.start_f.size();
  for (int s = 0; s < S; ++s) {
    path[s] = t.start_f[s];
    path[S + s] = t.end_f[s];
    path[2 * S + s] = t.start_b[s];
    path[3 * S + s] = t.end_b[s];
  }
}

// oldest entries no later plan depends on: executed, out of Q_train, not the last task, not the last training task
void prune(ls_node* n) {
  while (n->queue.size() > 1) {
    const PlannedTask& t = n->queue.front();
    if (!t.executed || t.in_train || t.id == n->last_train) break;
    n->queue.pop_front();
  }
}

}  // namespace

extern "C" {

ls_status ls_node_create(int S, double eta_f, double eta_b, ls_node** out) {
  LS_REQUIRE(out, "node_create: null output");
  LS_REQUIRE(S >= 1 && S <= 4096, "node_create: S = %d out of range", S);
  LS_REQUIRE(std::isfinite(eta_f) && std::isfinite(eta_b) && eta_f >= 0 && eta_b >= 0,
             "node_create: coefficients must be finite and non-negative");
  ls_node* n = new (std::nothrow) ls_node();
  if (!n) { ls_set_error("host allocation failed"); return LS_ENOMEM; }
  n->S = S;
  n->eta_f = eta_f;
  n->eta_b = eta_b;
  *out = n;
  return LS_OK;
}
void ls_node_destroy(ls_node* n) { delete n; }

ls_status ls_node_plan(ls_node* n, const ls_task* task, int commit, double* II, double* R, double* path,
                       int64_t* task_id) {
  LS_REQUIRE(n, "node_plan: null node");
  LS_REQUIRE(task_ok(task), "node_plan: task needs finite a and positive finite len and C");
  const int S = n->S;
  Plan p = compute_idleness(n, *task);
  if (II) *II = p.II;
  if (R) *R = p.R;
  PlannedTask t;
  t.id = -1;
  t.a = task->a; t.len = task->len; t.C = task->C;
  t.require_backward = task->require_backward != 0;
  t.in_train = false;
  t.executed = false;
  t.start_f = p.start_f;
  t.end_f = p.end_f;
  t.start_b.assign(S, 0.0);
  t.end_b.assign(S, 0.0);
  if (commit) {
    for (int64_t id : p.removed)
      if (PlannedTask* r = find_task(n, id)) r->in_train = false;
    if (t.require_backward) {
      const PlannedTask* before = n->last_train >= 0 ? find_task(n, n->last_train) : nullptr;
      const double delta_b = n->eta_b * t.C * t.len * t.len;
      double prev = t.end_f[S - 1];
      for (int s = S - 1; s >= 0; --s) {
        double start = prev;
        if (before) start = std::max(start, before->end_b[s]);
        t.start_b[s] = start;
        t.end_b[s] = start + delta_b;
        prev = t.end_b[s];
      }
      t.in_train = true;
    }
    t.id = n->next_id++;
    if (t.require_backward) n->last_train = t.id;
    n->lens.push_back(t.len);
    if (task_id) *task_id = t.id;
  }
  if (path) write_path(t, path);
  if (commit) n->queue.push_back(std::move(t));
  return LS_OK;
}

int ls_node_prune(ls_node* n) {
  if (!n) return 0;
  const size_t before = n->queue.size();
  prune(n);
  return (int)(before - n->queue.size());
}

int ls_node_queue_len(const ls_node* n, int train_only) {
  if (!n) return 0;
  if (!train_only) return (int)n->queue.size();
  int c = 0;
  for (const auto& t : n->queue) c += t.in_train;
  return c;
}

ls_status ls_node_task_path(const ls_node* n, int64_t task_id, double* path) {
  LS_REQUIRE(n && path, "node_task_path: null argument");
  const PlannedTask* t = find_task(n, task_id);
  LS_REQUIRE(t, "node_task_path: no task %lld in the trace queue", (long long)task_id);
  write_path(*t, path);
  return LS_OK;
}

ls_status ls_node_calibrate(ls_node* n, int64_t task_id, int stage, int backward, double start, double end) {
  LS_REQUIRE(n, "node_calibrate: null node");
  PlannedTask* t = find_task(n, task_id);
  LS_REQUIRE(t, "node_calibrate: no task %lld in the trace queue", (long long)task_id);
  LS_REQUIRE(stage >= 0 && stage < n->S, "node_calibrate: stage %d out of range", stage);
  LS_REQUIRE(!backward || t->require_backward, "node_calibrate: task %lld has no backward path", (long long)task_id);
  if (backward) { t->start_b[stage] = start; t->end_b[stage] = end; }
  else { t->start_f[stage] = start; t->end_f[stage] = end; }
  return LS_OK;
}

ls_status ls_node_score(ls_node* n, const ls_task* task, double a_prev, const ls_score_params* p, double* f,
                        double* IP, double* LC, double* II, double* R) {
  LS_REQUIRE(n && p, "node_score: null argument");
  LS_REQUIRE(task_ok(task), "node_score: task needs finite a and positive finite len and C");
  LS_REQUIRE(p->lambda1 > 0, "node_score: lambda1 must be positive");
  const Plan pl = compute_idleness(n, *task);
  const double ip = idleness_profit(pl.II, n->S, task->a, a_prev, p->tau);
  const double lc = length_consistency(n, task->len);
  if (II) *II = pl.II;
  if (R) *R = pl.R;
  if (IP) *IP = ip;
  if (LC) *LC = lc;
  if (f) *f = (ip + p->lambda2 * lc) / (p->lambda1 * pl.R);
  return LS_OK;
}

ls_status ls_select_node(ls_node* const* nodes, int N, const ls_task* task, double a_prev,
                         const ls_score_params* p, int* best, double* scores) {
  LS_REQUIRE(nodes && N >= 1 && best, "select_node: bad argument");
  int arg = -1;
  double top = 0.0;
  for (int i = 0; i < N; ++i) {
    double f;
    LS_TRY(ls_node_score(nodes[i], task, a_prev, p, &f, nullptr, nullptr, nullptr, nullptr));
    if (scores) scores[i] = f;
    if (arg < 0 || f > top) { arg = i; top = f; }
  }
  *best = arg;
  return LS_OK;
}

ls_status ls_deprioritize(ls_node* const* nodes, int N, const ls_task* next, double tau_R, int* deprioritize,
                          double* bound) {
  LS_REQUIRE(nodes && N >= 1, "deprioritize: bad argument");
  LS_REQUIRE(task_ok(next), "deprioritize: task needs finite a and positive finite len and C");
  double best = 0.0;
  for (int i = 0; i < N; ++i) {
    const ls_node* n = nodes[i];
    LS_REQUIRE(n, "deprioritize: null node %d", i);
    double latest = next->a;
    if (!n->queue.empty()) {
      latest = n->queue.front().end_f[n->S - 1];
      for (const auto& t : n->queue) latest = std::max(latest, t.end_f[n->S - 1]);
    }
    const double r = latest + n->eta_f * next->C * next->len * next->len - next->a;
    if (i == 0 || r < best) best = r;
  }
  if (bound) *bound = best;
  if (deprioritize) *deprioritize = best > tau_R ? 1 : 0;
  return LS_OK;
}

ls_status ls_node_execute(ls_node* n, double dt, double t_max, const ls_exec_hooks* h, ls_exec_stats* stats) {
  LS_REQUIRE(n && h, "node_execute: null argument");
  LS_REQUIRE(h->memory_available && h->wait && h->offload && h->forward && h->backward,
             "node_execute: every hook is required");
  LS_REQUIRE(dt > 0 && t_max >= 0, "node_execute: dt must be positive and t_max non-negative");
  ls_exec_stats st = {0, 0, 0, 0, 0, 0.0};
  const int S = n->S;
  std::vector<double> bs(S), be(S);
  for (;;) {
    // dequeue: the oldest committed task that has not run (ids are stable, the deque may be pruned)
    int64_t id = -1;
    for (const auto& t : n->queue)
      if (!t.executed) { id = t.id; break; }
    if (id < 0) break;
    ++st.tasks;
    const bool train = find_task(n, id)->require_backward;
    for (int s = 0; s < S; ++s) {
      double wait = 0.0;
      while (!h->memory_available(h->ctx, s)) {
        wait = wait + dt;
        st.waited += dt;
        h->wait(h->ctx, dt);
        if (wait >= t_max) {
          h->offload(h->ctx, id, s);
          ++st.offloads;
          break;
        }
      }
      if (h->memory_available(h->ctx, s)) {
        double a = 0, b = 0;
        h->forward(h->ctx, id, s, &a, &b);
        ++st.forwards;
        PlannedTask* t = find_task(n, id);
        t->start_f[s] = a;
        t->end_f[s] = b;
        if (s == S - 1 && train) {
          h->backward(h->ctx, id, bs.data(), be.data());
          ++st.backwards;
          t->start_b = bs;
          t->end_b = be;
        }
      } else {
        ++st.skipped_forwards;
      }
    }
    find_task(n, id)->executed = true;
  }
  if (stats) *stats = st;
  return LS_OK;
}

ls_status ls_batcher_create(int C, double T_w, ls_batcher** out) {
  LS_REQUIRE(out, "batcher_create: null output");
  LS_REQUIRE(C >= 1, "batcher_create: C must be at least 1");
  LS_REQUIRE(T_w >= 0, "batcher_create: T_w must be non-negative");
  ls_batcher* b = new (std::nothrow) ls_batcher();
  if (!b) { ls_set_error("host allocation failed"); return LS_ENOMEM; }
  b->C = C;
  b->T_w = T_w;
  *out = b;
  return LS_OK;
}
void ls_batcher_destroy(ls_batcher* b) { delete b; }

ls_status ls_batcher_push(ls_batcher* b, int64_t request_id, int require_backward) {
  LS_REQUIRE(b, "batcher_push: null batcher");
  LS_REQUIRE(request_id >= 0, "batcher_push: request ids are non-negative");
  b->queue.push_back({request_id, require_backward != 0});
  return LS_OK;
}

ls_status ls_batcher_form(ls_batcher* b, double now, int64_t* batch_ids, int* n_batch, int* n_new,
                          int* head_is_training) {
  LS_REQUIRE(b && batch_ids && n_batch, "batcher_form: null argument");
  if (b->batch.empty()) b->t_start = now;
  int added = 0, blocked = 0;
  while (!b->queue.empty() && (int)b->batch.size() < b->C) {
    const ls_batcher::Req& r = b->queue.front();
    if (!r.require_backward && b->t_start + b->T_w > now) {
      b->batch.push_back(r.id);
      b->queue.pop_front();
      ++added;
    } else {
      blocked = r.require_backward ? 1 : 0;
      break;
    }
  }
  for (size_t i = 0; i < b->batch.size(); ++i) batch_ids[i] = b->batch[i];
  *n_batch = (int)b->batch.size();
  if (n_new) *n_new = added;
  if (head_is_training) *head_is_training = blocked;
  return LS_OK;
}

ls_status ls_batcher_take_training(ls_batcher* b, int64_t* request_id) {
  LS_REQUIRE(b && request_id, "batcher_take_training: null argument");
  *request_id = -1;
  if (!b->queue.empty() && b->queue.front().require_backward) {
    *request_id = b->queue.front().id;
    b->queue.pop_front();
  }
  return LS_OK;
}

ls_status ls_batcher_finish(ls_batcher* b, const int64_t* finished_ids, int n) {
  LS_REQUIRE(b && (n == 0 || finished_ids) && n >= 0, "batcher_finish: bad argument");
  for (int i = 0; i < n; ++i) {
    auto it = std::find(b->batch.begin(), b->batch.end(), finished_ids[i]);
    if (it != b->batch.end()) b->batch.erase(it);
  }
  return LS_OK;
}

int ls_batcher_queued(const ls_batcher* b) { return b ? (int)b->queue.size() : 0; }
int ls_batcher_batch_size(const ls_batcher* b) { return b ? (int)b->batch.size() : 0; }

}  // extern "C"
