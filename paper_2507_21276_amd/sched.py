"""Python binding of the host scheduling steps (include/lemix_sched.h): argument marshalling
only, every decision is taken in the library."""
from __future__ import annotations

import ctypes as C

from . import binding as Bd


class ls_task(C.Structure):
    _fields_ = [("a", C.c_double), ("len", C.c_double), ("C", C.c_double), ("require_backward", C.c_int32)]


class ls_score_params(C.Structure):
    _fields_ = [("tau", C.c_double), ("lambda1", C.c_double), ("lambda2", C.c_double)]


class ls_exec_stats(C.Structure):
    _fields_ = [("tasks", C.c_int64), ("forwards", C.c_int64), ("backwards", C.c_int64),
                ("offloads", C.c_int64), ("skipped_forwards", C.c_int64), ("waited", C.c_double)]


_MEM = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_int)
_WAIT = C.CFUNCTYPE(None, C.c_void_p, C.c_double)
_OFF = C.CFUNCTYPE(None, C.c_void_p, C.c_int64, C.c_int)
_FWD = C.CFUNCTYPE(None, C.c_void_p, C.c_int64, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double))
_BWD = C.CFUNCTYPE(None, C.c_void_p, C.c_int64, C.POINTER(C.c_double), C.POINTER(C.c_double))


class ls_exec_hooks(C.Structure):
    _fields_ = [("ctx", C.c_void_p), ("memory_available", _MEM), ("wait", _WAIT), ("offload", _OFF),
                ("forward", _FWD), ("backward", _BWD)]


def _task(a, l, Cb, require_backward):
    return ls_task(float(a), float(l), float(Cb), int(bool(require_backward)))


class Node:
    """One node's trace queues (Algorithm 1, Eq. 1-4, Algorithm 2)."""

    def __init__(self, S, eta_f, eta_b):
        self.S = S
        self.h = C.c_void_p()
        self._destroy = Bd.lib().ls_node_destroy      # kept on the object: module globals may be gone at exit
        Bd._check(Bd.lib().ls_node_create(S, eta_f, eta_b, C.byref(self.h)))

    def __del__(self):
        if getattr(self, "h", None):
            self._destroy(self.h)
            self.h = None

    def plan(self, a, l, Cb, require_backward=False, commit=False):
        II, R, tid = C.c_double(), C.c_double(), C.c_int64(-1)
        path = (C.c_double * (4 * self.S))()
        t = _task(a, l, Cb, require_backward)
        Bd._check(Bd.lib().ls_node_plan(self.h, C.byref(t), int(commit), C.byref(II), C.byref(R), path,
                                        C.byref(tid)))
        S = self.S
        p = list(path)
        return dict(II=II.value, R=R.value, id=tid.value, start_f=p[:S], end_f=p[S:2 * S],
                    start_b=p[2 * S:3 * S], end_b=p[3 * S:])

    def path(self, task_id):
        path = (C.c_double * (4 * self.S))()
        Bd._check(Bd.lib().ls_node_task_path(self.h, task_id, path))
        S = self.S
        p = list(path)
        return dict(start_f=p[:S], end_f=p[S:2 * S], start_b=p[2 * S:3 * S], end_b=p[3 * S:])

    def calibrate(self, task_id, stage, backward, start, end):
        Bd._check(Bd.lib().ls_node_calibrate(self.h, task_id, stage, int(backward), start, end))

    def queue_len(self, train_only=False):
        return Bd.lib().ls_node_queue_len(self.h, int(train_only))

    def prune(self):
        return Bd.lib().ls_node_prune(self.h)

    def score(self, a, l, Cb, a_prev, tau, lambda1, lambda2):
        t = _task(a, l, Cb, False)
        p = ls_score_params(tau, lambda1, lambda2)
        out = [C.c_double() for _ in range(5)]
        Bd._check(Bd.lib().ls_node_score(self.h, C.byref(t), a_prev, C.byref(p), *[C.byref(o) for o in out]))
        return dict(zip(("f", "IP", "LC", "II", "R"), (o.value for o in out)))

    def execute(self, dt, t_max, memory_available, wait, offload, forward, backward):
        """Algorithm 2 with Python callables as hooks: memory_available(stage) -> bool,
        wait(seconds), offload(task_id, stage), forward(task_id, stage) -> (start, end),
        backward(task_id) -> (starts, ends)."""
        S = self.S

        def fwd(_, tid, s, ps, pe):
            ps[0], pe[0] = forward(tid, s)

        def bwd(_, tid, ps, pe):
            a, b = backward(tid)
            for i in range(S):
                ps[i], pe[i] = a[i], b[i]

        hooks = ls_exec_hooks(None, _MEM(lambda _, s: int(bool(memory_available(s)))),
                              _WAIT(lambda _, sec: wait(sec)), _OFF(lambda _, tid, s: offload(tid, s)),
                              _FWD(fwd), _BWD(bwd))
        st = ls_exec_stats()
        Bd._check(Bd.lib().ls_node_execute(self.h, dt, t_max, C.byref(hooks), C.byref(st)))
        return {k: getattr(st, k) for k, _ in ls_exec_stats._fields_}


def _handles(nodes):
    return (C.c_void_p * len(nodes))(*[n.h for n in nodes])


def select_node(nodes, a, l, Cb, a_prev, tau, lambda1, lambda2):
    t = _task(a, l, Cb, False)
    p = ls_score_params(tau, lambda1, lambda2)
    best = C.c_int(-1)
    scores = (C.c_double * len(nodes))()
    Bd._check(Bd.lib().ls_select_node(_handles(nodes), len(nodes), C.byref(t), a_prev, C.byref(p),
                                      C.byref(best), scores))
    return best.value, list(scores)


def deprioritize(nodes, a2, l2, C2, tau_R):
    t = _task(a2, l2, C2, False)
    flag, bound = C.c_int(0), C.c_double()
    Bd._check(Bd.lib().ls_deprioritize(_handles(nodes), len(nodes), C.byref(t), tau_R, C.byref(flag),
                                       C.byref(bound)))
    return bool(flag.value), bound.value


class Batcher:
    """Algorithm 3 (ContinuousBatching)."""

    def __init__(self, Cmax, T_w):
        self.C = Cmax
        self.h = C.c_void_p()
        self._destroy = Bd.lib().ls_batcher_destroy
        Bd._check(Bd.lib().ls_batcher_create(Cmax, T_w, C.byref(self.h)))

    def __del__(self):
        if getattr(self, "h", None):
            self._destroy(self.h)
            self.h = None

    def push(self, rid, require_backward=False):
        Bd._check(Bd.lib().ls_batcher_push(self.h, rid, int(bool(require_backward))))

    def form(self, now):
        ids = (C.c_int64 * self.C)()
        nb, nn, blocked = C.c_int(), C.c_int(), C.c_int()
        Bd._check(Bd.lib().ls_batcher_form(self.h, now, ids, C.byref(nb), C.byref(nn), C.byref(blocked)))
        batch = list(ids[:nb.value])
        return batch, batch[nb.value - nn.value:], bool(blocked.value)

    def take_training(self):
        rid = C.c_int64(-1)
        Bd._check(Bd.lib().ls_batcher_take_training(self.h, C.byref(rid)))
        return None if rid.value < 0 else rid.value

    def finish(self, ids):
        arr = (C.c_int64 * max(1, len(ids)))(*ids)
        Bd._check(Bd.lib().ls_batcher_finish(self.h, arr, len(ids)))

    def queued(self):
        return Bd.lib().ls_batcher_queued(self.h)

    def batch_size(self):
        return Bd.lib().ls_batcher_batch_size(self.h)


class ls_server_config(C.Structure):
    _fields_ = [("max_batch", C.c_int32), ("max_wait", C.c_double), ("n_pages", C.c_int32),
                ("max_pages_per_req", C.c_int32), ("max_chunk", C.c_int32), ("max_tokens", C.c_int32)]


class ls_pass_report(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("n_batch", "n_new", "n_decode", "n_prefill", "n_rows", "n_stalled",
                                         "n_finished", "free_pages", "unreserved_pages")]


class Server:
    """Continuous-batching loop of one stage (include/lemix_serve.h).  k_pool, v_pool, and every
    request's X and Y are torch tensors the caller keeps alive."""

    def __init__(self, stage, k_pool, v_pool, *, max_batch, max_wait, max_pages_per_req, max_chunk, max_tokens):
        self.stage, self.k_pool, self.v_pool = stage, k_pool, v_pool
        self.cfg = ls_server_config(max_batch, max_wait, k_pool.shape[1], max_pages_per_req, max_chunk,
                                    max_tokens)
        self.h = C.c_void_p()
        self._destroy = Bd.lib().ls_server_destroy
        Bd._check(Bd.lib().ls_server_create(stage.h, C.byref(self.cfg), k_pool.data_ptr(), v_pool.data_ptr(),
                                            C.byref(self.h)))
        self.workspace = stage.new_workspace(max_tokens)
        self._keep = {}

    def close(self):
        if getattr(self, "h", None):
            self._destroy(self.h)
            self.h = None

    __del__ = close

    def submit(self, rid, X, Y, prompt_len, n_decode):
        Bd._check(Bd.lib().ls_server_submit(self.h, rid, X.data_ptr(), Y.data_ptr(), prompt_len, n_decode))
        self._keep[rid] = (X, Y)

    def run_pass(self, now, stream=None):
        rep = ls_pass_report()
        ran = (C.c_int64 * self.cfg.max_batch)()
        fin = (C.c_int64 * self.cfg.max_batch)()
        Bd._check(Bd.lib().ls_server_pass(self.h, now, Bd._p(self.workspace), Bd._stream(stream), C.byref(rep),
                                          ran, fin))
        out = {k: getattr(rep, k) for k, _ in ls_pass_report._fields_}
        out["ran"] = list(ran[:rep.n_decode + rep.n_prefill])
        out["finished"] = list(fin[:rep.n_finished])
        return out

    def in_flight(self):
        return Bd.lib().ls_server_in_flight(self.h)
