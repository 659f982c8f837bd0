"""Pins for the scheduling oracle: values worked by hand from Algorithms 1-3 and Eq. 1-4, a
library density for Eq. 2, and a tick-by-tick pipeline simulation for the forward paths."""
import math

import pytest
from scipy.stats import norm

from oracle import sched_oracle as O


def approx(v):
    return pytest.approx(v, rel=1e-12, abs=1e-12)


# ---------------------------------------------------------------- Algorithm 1
def test_empty_node_pipeline_fill():
    # S = 3, delta_F = 1e-3 * 2 * 10^2 = 0.2, arrival 5: stage s starts when stage s-1 ends;
    # the idle time created before the task on stage s is (s-1) * delta_F
    n = O.Node(3, 1e-3, 0.0)
    II, R, sf, ef, rem = O.compute_idleness(n, 5.0, 10.0, 2.0)
    assert sf == approx([5.0, 5.2, 5.4]) and ef == approx([5.2, 5.4, 5.6])
    assert II == approx(0.6) and R == approx(0.6) and rem == []


def test_back_to_back_inference_creates_no_idleness():
    n = O.Node(3, 1e-3, 0.0)
    O.commit(n, 5.0, 10.0, 2.0, False)
    II, R, sf, ef, _ = O.compute_idleness(n, 5.0, 10.0, 2.0)
    assert sf == approx([5.2, 5.4, 5.6]) and ef == approx([5.4, 5.6, 5.8])
    assert II == approx(0.0) and R == approx(0.8)


def make_t1():
    # S = 2, eta_F = 1, eta_B = 2; training task a=0, l=1, C=1: forward [0,1],[1,2];
    # backward stage 2 [2,4], stage 1 [4,6]
    n = O.Node(2, 1.0, 2.0)
    t1, II, R = O.commit(n, 0.0, 1.0, 1.0, True)
    return n, t1


def test_training_task_paths():
    n, t1 = make_t1()
    assert t1.start_f == [0.0, 1.0] and t1.end_f == [1.0, 2.0]
    assert t1.start_b == [4.0, 2.0] and t1.end_b == [6.0, 4.0]
    assert n.train == [t1] and n.queue == [t1]


def test_forward_waits_for_a_backward_and_the_wait_is_not_idleness():
    # inference a=1, delta_F=1 after T1.  Stage 1: [1,2] ends before T1's backward there (4): fits.
    # Stage 2: [2,3] would overlap T1's backward [2,4] -> postponed to [4,5]; the backward ran
    # between the previous forward (ended 2) and this one, so its 2 s are subtracted: II = 0.
    n, t1 = make_t1()
    II, R, sf, ef, rem = O.compute_idleness(n, 1.0, 1.0, 1.0)
    assert sf == [1.0, 4.0] and ef == [2.0, 5.0]
    assert II == 0.0 and R == 4.0 and rem == []
    assert n.train == [t1]            # evaluation changes nothing
    # a third task behind it: prev_end = [2,5]; stage 2 starts at 5 after T1's backward ended
    # (4), no postponement beyond prev, no offset (prev ended after the backward started)
    O.commit(n, 1.0, 1.0, 1.0, False)
    II, R, sf, ef, rem = O.compute_idleness(n, 1.5, 1.0, 1.0)
    assert sf == [2.0, 5.0] and ef == [3.0, 6.0] and II == 0.0 and R == 4.5 and rem == []


def test_long_forward_is_postponed_behind_the_backward_at_stage_one():
    # a=3, l=2 -> delta_F = 4.  Stage 1: [3,7] overlaps T1's backward [4,6] -> [6,10], offset 2,
    # T1 leaves Q_train (its backward path ends at stage 1).  II_1 = 6 - 1 - 2 = 3.
    # Stage 2: Q_temp is empty; start = max(10, 2) = 10; II_2 = 10 - 2 = 8.
    n, t1 = make_t1()
    II, R, sf, ef, rem = O.compute_idleness(n, 3.0, 2.0, 1.0)
    assert sf == [6.0, 10.0] and ef == [10.0, 14.0]
    assert II == 11.0 and R == 11.0 and rem == [t1]
    O.commit(n, 3.0, 2.0, 1.0, False)
    assert n.train == []


def test_second_training_task_backward_chains_behind_the_first():
    # T2 = T1's twin.  Forward: stage 1 [1,2] (fits before 4); stage 2 postponed to [4,5], offset 2.
    # Backward: stage 2 start max(5, T1.end_b=4) = 5 -> 7; stage 1 start max(7, 6) = 7 -> 9.
    n, t1 = make_t1()
    t2, II, R = O.commit(n, 0.0, 1.0, 1.0, True)
    assert t2.start_f == [1.0, 4.0] and t2.end_f == [2.0, 5.0] and II == 0.0 and R == 5.0
    assert t2.start_b == [7.0, 5.0] and t2.end_b == [9.0, 7.0]
    assert n.train == [t1, t2]


def simulate_fifo_pipeline(tasks, S):
    """Integer-time simulation of S servers in a line, each serving tasks in arrival order."""
    n = len(tasks)
    done = [[None] * S for _ in range(n)]
    start = [[None] * S for _ in range(n)]
    busy_until = [0] * S
    nxt = [0] * S
    t = 0
    while any(d[S - 1] is None for d in done):
        for s in range(S):
            i = nxt[s]
            if i >= n or busy_until[s] > t:
                continue
            ready = tasks[i][0] if s == 0 else done[i][s - 1]
            if ready is not None and ready <= t:
                start[i][s] = t
                done[i][s] = t + tasks[i][1]
                busy_until[s] = done[i][s]
                nxt[s] += 1
        t += 1
    return start, done


def test_inference_only_paths_match_a_pipeline_simulation():
    # arrival, duration (integers); eta_F = 1, C = duration, l = 1
    tasks = [(0, 3), (1, 1), (2, 5), (20, 2), (21, 2), (21, 4), (40, 1)]
    S = 4
    start, done = simulate_fifo_pipeline(tasks, S)
    n = O.Node(S, 1.0, 0.0)
    for i, (a, p) in enumerate(tasks):
        t, II, R = O.commit(n, float(a), 1.0, float(p), False)
        assert t.start_f == [float(x) for x in start[i]]
        assert t.end_f == [float(x) for x in done[i]]
        assert R == done[i][S - 1] - a
        # without training tasks II is the gap each stage sat idle in front of this task
        prev = done[i - 1] if i else [a] * S
        assert II == sum(start[i][s] - prev[s] for s in range(S))


# ------------------------------------------------------------------- Eq. 1-4
def test_idleness_profit():
    assert O.idleness_profit(11.0, 2, 3.0, 1.0, -1.0) == -3.5     # 11/2 - 2 = 3.5 > tau
    assert O.idleness_profit(11.0, 2, 3.0, 1.0, 5.0) == -5.0      # tau floors the penalty
    assert O.idleness_profit(0.0, 4, 9.0, 1.0, -2.0) == 2.0       # -8 < tau = -2


def test_length_consistency_is_the_normal_density_of_the_history():
    lens = [100.0, 220.0, 130.0, 512.0, 64.0]
    mu = sum(lens) / 5
    sigma = math.sqrt(sum((x - mu) ** 2 for x in lens) / 5)
    for l in (64.0, 200.0, 900.0):
        assert O.length_consistency(l, lens) == approx(norm.pdf(l, loc=mu, scale=sigma))
    assert O.length_consistency(10.0, []) == 0.0
    assert O.length_consistency(10.0, [10.0]) == 0.0
    assert O.length_consistency(10.0, [10.0, 10.0]) == 0.0


def test_node_priority_and_selection():
    assert O.node_priority(-3.5, 0.25, 11.0, 2.0, 4.0) == approx((-3.5 + 1.0) / 22.0)
    # two nodes, S = 2, eta_F = 1: node 0 holds T1 (see above), node 1 is empty.
    # task a=3, l=2, C=1, a_prev=1, tau=-10, lambda1=1, lambda2=0:
    #   node 0: II=11, R=11 -> IP = -(5.5 - 2) = -3.5, f = -3.5/11
    #   node 1: II = 0 + 4, R = 8 -> IP = -(2 - 2) = 0 -> f = 0
    n0, _ = make_t1()
    n1 = O.Node(2, 1.0, 2.0)
    best, fs = O.select_node([n0, n1], 3.0, 2.0, 1.0, 1.0, -10.0, 1.0, 0.0)
    assert fs == approx([-3.5 / 11.0, 0.0]) and best == 1
    # ties go to the first node
    best, fs = O.select_node([O.Node(2, 1.0, 2.0), O.Node(2, 1.0, 2.0)], 3.0, 2.0, 1.0, 1.0, -10.0, 1.0, 0.0)
    assert best == 0


def test_response_bound_and_deprioritisation():
    # node A: tasks whose last-stage forward ends at 5 and 14; node B empty; eta_F = 1.
    # next inference a'=3, C'=1, l'=2: A -> 14 + 4 - 3 = 15, B -> 3 + 4 - 3 = 4; min = 4
    A = O.Node(2, 1.0, 2.0)
    O.commit(A, 0.0, 1.0, 1.0, True)          # ends forward at 2
    O.commit(A, 3.0, 2.0, 1.0, False)         # ends forward at 14 (worked example above)
    B = O.Node(2, 1.0, 2.0)
    assert O.response_bound([A], 3.0, 2.0, 1.0) == 15.0
    assert O.response_bound([A, B], 3.0, 2.0, 1.0) == 4.0
    assert O.deprioritize([A, B], 3.0, 2.0, 1.0, 3.9)
    assert not O.deprioritize([A, B], 3.0, 2.0, 1.0, 4.0)


# ---------------------------------------------------------------- Algorithm 2
class ScriptedHooks:
    def __init__(self, avail):
        self.avail = list(avail)   # answers of MemoryAvailable, in call order; last one repeats
        self.calls = []
        self.clock = 0.0

    def memory_available(self, s):
        v = self.avail.pop(0) if len(self.avail) > 1 else self.avail[0]
        self.calls.append(("mem", s, v))
        return v

    def wait(self, dt):
        self.clock += dt

    def offload(self, task, s):
        self.calls.append(("offload", task.id, s))

    def forward(self, task, s):
        self.clock += 1.0
        return self.clock - 1.0, self.clock

    def backward(self, task):
        S = len(task.start_f)
        out = [(self.clock + (S - 1 - s), self.clock + (S - s)) for s in range(S)]
        self.clock += S
        return [o[0] for o in out], [o[1] for o in out]


def test_wait_then_run():
    n = O.Node(2, 1.0, 2.0)
    O.commit(n, 0.0, 1.0, 1.0, True)
    # stage 0: unavailable twice, then available (loop check, then the check before Forward);
    # stage 1: available at once
    h = ScriptedHooks([False, False, True, True, True, True])
    log = O.execute_memory_aware(n, h, 0.1, 0.25)
    assert log == [("forward", 0, 0), ("forward", 0, 1), ("backward", 0)]
    assert h.clock == approx(0.2 + 1.0 + 1.0 + 2.0)
    t = n.queue[0]
    assert t.start_f == approx([0.2, 1.2]) and t.end_f == approx([1.2, 2.2])      # calibrated
    assert t.start_b == approx([3.2, 2.2]) and t.end_b == approx([4.2, 3.2])
    assert n.pending == []


def test_wait_reaches_t_max_then_offload_and_skip():
    n = O.Node(2, 1.0, 2.0)
    O.commit(n, 0.0, 1.0, 1.0, False)
    # never available at stage 0: three waits of 0.1 reach T_max = 0.25 -> offload; still not
    # available -> that stage's forward is skipped; stage 1 then runs
    h = ScriptedHooks([False, False, False, False, True, True])
    log = O.execute_memory_aware(n, h, 0.1, 0.25)
    assert log == [("offload", 0, 0), ("skip", 0, 0), ("forward", 0, 1)]
    assert [c for c in h.calls if c[0] == "offload"] == [("offload", 0, 0)]
    assert h.clock == approx(0.3 + 1.0)


# ---------------------------------------------------------------- Algorithm 3
def test_batcher_fcfs_up_to_c():
    b = O.Batcher(2, 0.5)
    for i in range(3):
        b.push(i, False)
    assert b.form(0.0) == ([0, 1], [0, 1], False)
    assert b.form(0.1) == ([0, 1], [], False)          # full
    b.finish([0])
    assert b.form(0.2) == ([1, 2], [2], False)          # batch not empty: T_start stays 0.0


def test_batcher_wait_limit():
    b = O.Batcher(4, 0.5)
    b.push(0, False)
    assert b.form(1.0) == ([0], [0], False)             # T_start = 1.0
    b.push(1, False)
    assert b.form(1.4) == ([0, 1], [1], False)          # 1.0 + 0.5 > 1.4
    b.push(2, False)
    assert b.form(1.5) == ([0, 1], [], False)           # 1.0 + 0.5 > 1.5 fails: not admitted
    b.finish([0, 1])
    assert b.form(1.6) == ([2], [2], False)             # empty batch: T_start = 1.6


def test_batcher_training_task_at_the_head_ends_the_round():
    b = O.Batcher(4, 0.5)
    b.push(0, False)
    b.push(1, True)
    b.push(2, False)
    assert b.form(0.0) == ([0], [0], True)
    assert b.take_training() == 1
    assert b.take_training() is None
    assert b.form(0.1) == ([0, 2], [2], False)
