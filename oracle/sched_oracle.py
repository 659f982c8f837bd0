"""CPU oracle for the host-side scheduling steps around the stage.  TEST INFRASTRUCTURE.

Only tests may import this file; it shares no code with the package.  Plain Python, the
algorithms' steps in the paper's order and notation:

  compute_idleness      Algorithm 1 (ComputeIdleness): forward path of a new task on a node,
                        idleness increased II and response time R
  plan_backward         "Backward planning" paragraph of Task-Specific Execution Planning
  idleness_profit       Eq. 1      length_consistency   Eq. 2      node_priority   Eq. 3
  select_node           task-level allocation: the node with the highest priority score
  response_bound        left-hand side of Eq. 4 (queue-level deprioritisation of training tasks)
  execute_memory_aware  Algorithm 2 (ExecuteTaskMemoryAware): wait-or-drop, calibration
  Batcher               Algorithm 3 (ContinuousBatching): FCFS admission with C and T_w

Stages are 0-based here (the paper's stage s is index s - 1).  Times are plain floats.

Readings where the paper is silent or its listing is ambiguous:
  S1  end_f of "stage 0" of the new task is its arrival time a.
  S2  on a node with an empty trace queue task_prev.end_f is a at every stage.
  S3  Q_temp is filled once, before the stage loop, from Q_train in enqueue order.  A training
      task the forward fits in front of goes back to the head of Q_temp; one that postpones the
      forward is consumed and is not seen by later stages.
  S4  CheckExecuted(t, 1): t's backward at the first stage (the last one of its backward path)
      ends no later than the new task's forward start there, which always holds after the
      postponement; t then leaves Q_train.  Evaluating a node for a task changes nothing; the
      removal is applied when the task is committed to that node.
  S5  backward path: start_b at the last stage is max(end_f there, end_b there of the last
      training task committed before); going down, start_b[s] = max(end_b[s + 1], that task's
      end_b[s]); end_b = start_b + eta_B C l^2.
  S6  Eq. 2 with fewer than two executed tasks, or sigma = 0, gives LC = 0; sigma is the
      population standard deviation.
  S7  Eq. 4: the inner maximum runs over the tasks queued on the node (their forward end at the
      last stage) and is a' on an empty node.  The training task is deprioritised when the
      bound is strictly greater than tau_R.
  S8  Algorithm 3 looks at the head of the queue without removing it; a request is removed when
      it joins the batch.  A training task at the head ends the admission round and stays
      there until the caller takes it.
"""
import math


class Task:
    def __init__(self, a, l, C, require_backward, S):
        self.a, self.l, self.C, self.require_backward = a, l, C, bool(require_backward)
        self.start_f, self.end_f = [0.0] * S, [0.0] * S
        self.start_b, self.end_b = [0.0] * S, [0.0] * S
        self.id = -1


class Node:
    def __init__(self, S, eta_f, eta_b):
        self.S, self.eta_f, self.eta_b = S, eta_f, eta_b
        self.queue = []      # Q^n: every committed task, in enqueue order
        self.train = []      # Q^n_train: training tasks whose backward may still interfere
        self.pending = []    # committed, not yet executed (Algorithm 2 takes from here)
        self.lens = []       # query lengths of the tasks given to the node (Eq. 2)
        self.last_train = None
        self.next_id = 0


def compute_idleness(node, a, l, C):
    """Algorithm 1.  Returns (II, R, start_f, end_f, removed): removed lists the training
    tasks that CheckExecuted takes out of Q_train (reading S4)."""
    S = node.S
    delta_f = node.eta_f * C * l * l
    prev_end = list(node.queue[-1].end_f) if node.queue else [a] * S
    q_temp = list(node.train)
    removed = []
    II = 0.0
    start_f, end_f = [0.0] * S, [0.0] * S
    end_before = a
    for s in range(S):
        start = max(end_before, prev_end[s])
        end = start + delta_f
        offset = 0.0
        while q_temp:
            t = q_temp.pop(0)
            if end <= t.start_b[s]:
                q_temp.insert(0, t)
                break
            start = max(start, t.end_b[s])
            end = start + delta_f
            if prev_end[s] <= t.start_b[s]:
                offset = offset + node.eta_b * t.C * t.l * t.l
            if s == 0:
                removed.append(t)
        II = II + start - prev_end[s] - offset
        start_f[s], end_f[s] = start, end
        end_before = end
    R = end_f[S - 1] - a
    return II, R, start_f, end_f, removed


def plan_backward(node, task):
    S = node.S
    delta_b = node.eta_b * task.C * task.l * task.l
    before = task.end_f[S - 1]
    for s in range(S - 1, -1, -1):
        start = before
        if node.last_train is not None:
            start = max(start, node.last_train.end_b[s])
        task.start_b[s] = start
        task.end_b[s] = start + delta_b
        before = task.end_b[s]


def commit(node, a, l, C, require_backward):
    """Plans the task on the node (Algorithm 1, then the backward path) and enqueues it."""
    II, R, start_f, end_f, removed = compute_idleness(node, a, l, C)
    t = Task(a, l, C, require_backward, node.S)
    t.start_f, t.end_f = start_f, end_f
    t.id = node.next_id
    node.next_id += 1
    for r in removed:
        node.train.remove(r)
    if t.require_backward:
        plan_backward(node, t)
        node.train.append(t)
        node.last_train = t
    node.queue.append(t)
    node.pending.append(t)
    node.lens.append(l)
    return t, II, R


def idleness_profit(II, S, a, a_prev, tau):
    return -max(II / S - (a - a_prev), tau)


def length_consistency(l, lens):
    n = len(lens)
    if n < 2:
        return 0.0
    mu = sum(lens) / n
    var = sum((x - mu) * (x - mu) for x in lens) / n
    if var <= 0.0:
        return 0.0
    sigma = math.sqrt(var)
    return 1.0 / (sigma * math.sqrt(2.0 * math.pi)) * math.exp(-(l - mu) * (l - mu) / (2.0 * var))


def node_priority(IP, LC, R, lambda1, lambda2):
    return (IP + lambda2 * LC) / (lambda1 * R)


def score(node, a, l, C, a_prev, tau, lambda1, lambda2):
    II, R, _, _, _ = compute_idleness(node, a, l, C)
    IP = idleness_profit(II, node.S, a, a_prev, tau)
    LC = length_consistency(l, node.lens)
    return node_priority(IP, LC, R, lambda1, lambda2), IP, LC, II, R


def select_node(nodes, a, l, C, a_prev, tau, lambda1, lambda2):
    best, best_f, fs = -1, 0.0, []
    for i, n in enumerate(nodes):
        f = score(n, a, l, C, a_prev, tau, lambda1, lambda2)[0]
        fs.append(f)
        if best < 0 or f > best_f:
            best, best_f = i, f
    return best, fs


def response_bound(nodes, a2, l2, C2):
    best = None
    for n in nodes:
        latest = a2
        if n.queue:
            latest = max(t.end_f[n.S - 1] for t in n.queue)
        r = latest + n.eta_f * C2 * l2 * l2 - a2
        if best is None or r < best:
            best = r
    return best


def deprioritize(nodes, a2, l2, C2, tau_R):
    return response_bound(nodes, a2, l2, C2) > tau_R


def execute_memory_aware(node, hooks, dt, t_max):
    """Algorithm 2.  hooks: memory_available(stage) -> bool, wait(seconds), offload(task, stage),
    forward(task, stage) -> (start, end), backward(task) -> (starts, ends).  Returns the log."""
    log = []
    while node.pending:
        task = node.pending.pop(0)
        for s in range(node.S):
            wait = 0.0
            while not hooks.memory_available(s):
                wait = wait + dt
                hooks.wait(dt)
                if wait >= t_max:
                    hooks.offload(task, s)
                    log.append(("offload", task.id, s))
                    break
            if hooks.memory_available(s):
                task.start_f[s], task.end_f[s] = hooks.forward(task, s)
                log.append(("forward", task.id, s))
                if s == node.S - 1 and task.require_backward:
                    starts, ends = hooks.backward(task)
                    task.start_b, task.end_b = list(starts), list(ends)
                    log.append(("backward", task.id))
            else:
                log.append(("skip", task.id, s))
    return log


class Batcher:
    """Algorithm 3: the batch-forming part of one pass of its outer loop (form), and the
    filter of finished requests after the batch ran (finish)."""

    def __init__(self, C, T_w):
        self.C, self.T_w = C, T_w
        self.queue = []      # (id, require_backward), FCFS
        self.batch = []
        self.t_start = 0.0

    def push(self, rid, require_backward):
        self.queue.append((rid, bool(require_backward)))

    def form(self, now):
        if not self.batch:
            self.t_start = now
        new, blocked = [], False
        while self.queue and len(self.batch) < self.C:
            rid, rb = self.queue[0]
            if (not rb) and self.t_start + self.T_w > now:
                self.queue.pop(0)
                self.batch.append(rid)
                new.append(rid)
            else:
                blocked = rb
                break
        return list(self.batch), new, blocked

    def take_training(self):
        if self.queue and self.queue[0][1]:
            return self.queue.pop(0)[0]
        return None

    def finish(self, ids):
        gone = set(ids)
        self.batch = [b for b in self.batch if b not in gone]
