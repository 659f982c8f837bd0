"""The library's host scheduling steps against the plain-Python oracle, on seeded random traces
(CPU only: no call here touches the GPU)."""
import numpy as np
import pytest

from oracle import sched_oracle as O
from paper_2507_21276_amd import binding as Bd
from paper_2507_21276_amd import sched as Sc


def close(a, b):
    return a == pytest.approx(b, rel=1e-12, abs=1e-12)


def same_path(p, t):
    return (close(p["start_f"], t.start_f) and close(p["end_f"], t.end_f)
            and close(p["start_b"], t.start_b) and close(p["end_b"], t.end_b))


@pytest.mark.parametrize("seed,S,integer", [(1, 1, True), (2, 2, True), (3, 4, True), (4, 3, False), (5, 8, False)])
def test_planning_matches_the_oracle_on_random_traces(seed, S, integer):
    rng = np.random.default_rng(seed)
    eta_f, eta_b = (1.0, 2.0) if integer else (3.1e-7, 7.7e-7)
    n_lib, n_or = Sc.Node(S, eta_f, eta_b), O.Node(S, eta_f, eta_b)
    a = 0.0
    for i in range(200):
        a += float(rng.integers(0, 6)) if integer else float(rng.exponential(0.05))
        l = float(rng.integers(1, 4)) if integer else float(rng.integers(16, 2048))
        Cb = float(rng.integers(1, 3))
        rb = bool(rng.random() < 0.35)
        # evaluation changes nothing and agrees
        II, R, sf, ef, _ = O.compute_idleness(n_or, a, l, Cb)
        p = n_lib.plan(a, l, Cb, rb, commit=False)
        assert close(p["II"], II) and close(p["R"], R) and close(p["start_f"], sf) and close(p["end_f"], ef)
        assert n_lib.queue_len() == len(n_or.queue)
        t, II2, R2 = O.commit(n_or, a, l, Cb, rb)
        p = n_lib.plan(a, l, Cb, rb, commit=True)
        assert p["id"] == t.id and close(p["II"], II2) and close(p["R"], R2) and same_path(p, t)
        assert n_lib.queue_len(True) == len(n_or.train)
        assert same_path(n_lib.path(t.id), t)
    assert len(n_or.train) < 200    # the traces do exercise the removal from Q_train


@pytest.mark.parametrize("seed", [11, 12])
def test_scores_selection_and_deprioritisation_match_the_oracle(seed):
    rng = np.random.default_rng(seed)
    S, N = 3, 4
    etas = [(2e-7 * (1 + i), 5e-7 * (1 + i)) for i in range(N)]
    lib_nodes = [Sc.Node(S, *e) for e in etas]
    or_nodes = [O.Node(S, *e) for e in etas]
    tau, lam1, lam2 = -0.05, 1.5, 40.0
    a = a_prev = 0.0
    picks = []
    for i in range(150):
        a_prev, a = a, a + float(rng.exponential(0.02))
        l, Cb, rb = float(rng.integers(32, 1024)), float(rng.integers(1, 5)), bool(rng.random() < 0.3)
        for ln, on in zip(lib_nodes, or_nodes):
            f, IP, LC, II, R = O.score(on, a, l, Cb, a_prev, tau, lam1, lam2)
            s = ln.score(a, l, Cb, a_prev, tau, lam1, lam2)
            assert close(s["f"], f) and close(s["IP"], IP) and close(s["LC"], LC) and close(s["II"], II) and close(s["R"], R)
        best_o, fs_o = O.select_node(or_nodes, a, l, Cb, a_prev, tau, lam1, lam2)
        best_l, fs_l = Sc.select_node(lib_nodes, a, l, Cb, a_prev, tau, lam1, lam2)
        assert best_l == best_o and close(fs_l, fs_o)
        picks.append(best_o)
        O.commit(or_nodes[best_o], a, l, Cb, rb)
        lib_nodes[best_l].plan(a, l, Cb, rb, commit=True)
        a2, l2, C2 = a + 0.001, float(rng.integers(32, 1024)), 1.0
        bound = O.response_bound(or_nodes, a2, l2, C2)
        for tau_R in (bound * 0.5, bound * 2.0):
            flag, b = Sc.deprioritize(lib_nodes, a2, l2, C2, tau_R)
            assert close(b, bound) and flag == O.deprioritize(or_nodes, a2, l2, C2, tau_R)
    assert len(set(picks)) > 1        # the score does spread the work over nodes


class Script:
    """Scripted stand-ins for the stage: memory answers from a seeded stream, a clock that the
    forward, backward and wait hooks advance."""

    def __init__(self, seed, S, p_free):
        self.rng = np.random.default_rng(seed)
        self.S, self.p_free, self.clock, self.log = S, p_free, 0.0, []

    def memory_available(self, s):
        return bool(self.rng.random() < self.p_free)

    def wait(self, sec):
        self.clock += sec

    def offload(self, tid, s):
        self.log.append(("offload", tid, s))

    def forward(self, tid, s):
        self.log.append(("forward", tid, s))
        self.clock += 0.25
        return self.clock - 0.25, self.clock

    def backward(self, tid):
        self.log.append(("backward", tid))
        st = [self.clock + 0.5 * (self.S - 1 - s) for s in range(self.S)]
        self.clock += 0.5 * self.S
        return st, [x + 0.5 for x in st]


@pytest.mark.parametrize("seed,p_free", [(21, 0.9), (22, 0.3), (23, 0.05)])
def test_memory_aware_execution_matches_the_oracle(seed, p_free):
    S = 3
    n_lib, n_or = Sc.Node(S, 1e-6, 2e-6), O.Node(S, 1e-6, 2e-6)
    rng = np.random.default_rng(seed)
    tasks = [(0.1 * i, float(rng.integers(16, 512)), 2.0, bool(rng.random() < 0.4)) for i in range(40)]
    for t in tasks:
        O.commit(n_or, *t)
        n_lib.plan(*t, commit=True)
    h_or, h_lib = Script(seed, S, p_free), Script(seed, S, p_free)

    class OrHooks:
        memory_available = staticmethod(h_or.memory_available)
        wait = staticmethod(h_or.wait)
        offload = staticmethod(lambda task, s: h_or.offload(task.id, s))
        forward = staticmethod(lambda task, s: h_or.forward(task.id, s))
        backward = staticmethod(lambda task: h_or.backward(task.id))

    log = O.execute_memory_aware(n_or, OrHooks, 0.01, 0.035)
    stats = n_lib.execute(0.01, 0.035, h_lib.memory_available, h_lib.wait, h_lib.offload, h_lib.forward,
                          h_lib.backward)
    assert h_lib.log == h_or.log and close(h_lib.clock, h_or.clock)
    assert stats["tasks"] == 40
    assert stats["forwards"] == sum(e[0] == "forward" for e in log)
    assert stats["backwards"] == sum(e[0] == "backward" for e in log)
    assert stats["offloads"] == sum(e[0] == "offload" for e in log)
    assert stats["skipped_forwards"] == sum(e[0] == "skip" for e in log)
    if p_free < 0.5:
        assert stats["offloads"] > 0 and stats["skipped_forwards"] > 0
    for t in n_or.queue:                      # calibrated intervals
        assert same_path(n_lib.path(t.id), t)
    # planning after calibration still agrees, and pruning does not change what is planned
    II, R, sf, ef, _ = O.compute_idleness(n_or, 50.0, 100.0, 2.0)
    p = n_lib.plan(50.0, 100.0, 2.0)
    assert close(p["II"], II) and close(p["R"], R) and close(p["end_f"], ef)
    dropped = n_lib.prune()
    assert dropped > 0 and n_lib.queue_len() == 40 - dropped
    p2 = n_lib.plan(50.0, 100.0, 2.0)
    assert p2["II"] == p["II"] and p2["R"] == p["R"] and p2["end_f"] == p["end_f"]
    assert n_lib.execute(0.01, 0.035, h_lib.memory_available, h_lib.wait, h_lib.offload, h_lib.forward,
                         h_lib.backward)["tasks"] == 0


@pytest.mark.parametrize("seed,Cmax,T_w", [(31, 1, 0.2), (32, 4, 0.3), (33, 8, 0.05), (34, 64, 10.0)])
def test_batcher_matches_the_oracle(seed, Cmax, T_w):
    rng = np.random.default_rng(seed)
    b_lib, b_or = Sc.Batcher(Cmax, T_w), O.Batcher(Cmax, T_w)
    now, rid, left = 0.0, 0, {}
    admitted = 0
    for it in range(400):
        for _ in range(int(rng.integers(0, 3))):
            rb = bool(rng.random() < 0.15)
            b_lib.push(rid, rb)
            b_or.push(rid, rb)
            left[rid] = int(rng.integers(1, 6))
            rid += 1
        got, want = b_lib.form(now), b_or.form(now)
        assert got == want
        admitted += len(want[1])
        if want[2] or it % 7 == 0:       # also when the round did not stop at a training task
            assert b_lib.take_training() == b_or.take_training()
        done = []
        for r in want[0]:
            left[r] -= 1
            if left[r] == 0:
                done.append(r)
        b_lib.finish(done)
        b_or.finish(done)
        assert b_lib.batch_size() == len(b_or.batch) and b_lib.queued() == len(b_or.queue)
        now += float(rng.exponential(0.1))
    assert admitted > 50


def test_argument_errors():
    with pytest.raises(Bd.LsError):
        Sc.Node(0, 1.0, 1.0)
    with pytest.raises(Bd.LsError):
        Sc.Node(2, -1.0, 1.0)
    n = Sc.Node(2, 1.0, 1.0)
    with pytest.raises(Bd.LsError):
        n.plan(0.0, 0.0, 1.0)
    with pytest.raises(Bd.LsError):
        n.plan(float("nan"), 1.0, 1.0)
    with pytest.raises(Bd.LsError):
        n.path(7)
    tid = n.plan(0.0, 1.0, 1.0, False, commit=True)["id"]
    with pytest.raises(Bd.LsError):
        n.calibrate(tid, 2, False, 0.0, 1.0)
    with pytest.raises(Bd.LsError):
        n.calibrate(tid, 0, True, 0.0, 1.0)       # an inference task has no backward path
    with pytest.raises(Bd.LsError):
        n.score(0.0, 1.0, 1.0, 0.0, 0.0, 0.0, 1.0)  # lambda1 must be positive
    with pytest.raises(Bd.LsError):
        Sc.Batcher(0, 1.0)
    with pytest.raises(Bd.LsError):
        Sc.Batcher(2, -1.0)
