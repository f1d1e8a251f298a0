"""ctypes binding of the host-side schedule generator / performance model
(include/crosspipe_sched.h): same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
from typing import List, Sequence, Tuple

from . import stage as S

F, D, W = 0, 1, 2
E_INVAL, E_DEADLOCK = -1, -5


class Params(C.Structure):
    _fields_ = [("n_pp", C.c_int32), ("n_mb", C.c_int32), ("n_sub", C.c_int32),
                ("t_f", C.POINTER(C.c_double)), ("t_d", C.POINTER(C.c_double)), ("t_w", C.POINTER(C.c_double)),
                ("m_f", C.c_double), ("m_d", C.c_double), ("m_w", C.c_double), ("m_limit", C.c_double),
                ("alpha", C.POINTER(C.c_double)), ("beta", C.POINTER(C.c_double)), ("msg_bytes", C.c_double)]


class Slot(C.Structure):
    _fields_ = [("stage", C.c_int32), ("kind", C.c_int32), ("mb", C.c_int32), ("sub", C.c_int32),
                ("t_start", C.c_double), ("t_end", C.c_double)]

    def astuple(self):
        return (self.stage, self.kind, self.mb, self.sub, self.t_start, self.t_end)


_bound = False


def _lib():
    global _bound
    L = S.lib()
    if not _bound:
        pp, sp = C.POINTER(Params), C.POINTER(Slot)
        L.crosspipe_greedy.restype = C.c_int
        L.crosspipe_greedy.argtypes = [pp, sp, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_double)]
        L.crosspipe_simulate.restype = C.c_int
        L.crosspipe_simulate.argtypes = [pp, sp, C.c_int, sp, C.POINTER(C.c_double)]
        L.crosspipe_stage_ops.restype = C.c_int
        L.crosspipe_stage_ops.argtypes = [sp, C.c_int, C.c_int, C.POINTER(S.StageSubOp), C.c_int, C.POINTER(C.c_int)]
        _bound = True
    return L


def make_params(n_pp, n_mb, n_sub, t_f, t_d, t_w, m_f=1.0, m_d=0.0, m_w=-1.0, m_limit=1e30, alpha=None, beta=None,
                msg_bytes=0.0):
    """alpha / beta: n_pp x n_pp nested sequences or None. Returns (Params, keepalive)."""
    arr = lambda v: (C.c_double * len(v))(*v)
    flat = lambda m: arr([x for row in m for x in row]) if m is not None else None
    keep = [arr(list(t_f)), arr(list(t_d)), arr(list(t_w)), flat(alpha), flat(beta)]
    p = Params(n_pp, n_mb, n_sub, keep[0], keep[1], keep[2], m_f, m_d, m_w, m_limit,
               keep[3] if keep[3] is not None else None, keep[4] if keep[4] is not None else None, msg_bytes)
    return p, keep


def crosspipe_greedy(p: Params) -> Tuple[List[tuple], float]:
    n = 3 * p.n_mb * p.n_sub * p.n_pp
    out = (Slot * n)()
    cnt, mk = C.c_int(), C.c_double()
    rc = _lib().crosspipe_greedy(C.byref(p), out, n, C.byref(cnt), C.byref(mk))
    if rc:
        raise RuntimeError(f"crosspipe_greedy failed ({rc})")
    return [out[i].astuple() for i in range(cnt.value)], mk.value


def crosspipe_simulate(p: Params, per_stage: Sequence[Sequence[Tuple[int, int, int]]]) -> Tuple[int, List[tuple], float]:
    """per_stage[s]: ordered (kind, mb, sub). Returns (code, timed slots, makespan)."""
    flat = [(s, k, m, sb) for s, lst in enumerate(per_stage) for (k, m, sb) in lst]
    n = len(flat)
    inp, out = (Slot * max(1, n))(), (Slot * max(1, n))()
    for i, (s, k, m, sb) in enumerate(flat):
        inp[i] = Slot(s, k, m, sb, 0.0, 0.0)
    mk = C.c_double()
    rc = _lib().crosspipe_simulate(C.byref(p), inp, n, out, C.byref(mk))
    return rc, [out[i].astuple() for i in range(n)] if rc == 0 else [], mk.value


def crosspipe_stage_ops(slots: Sequence[tuple], stage: int) -> List[Tuple[int, int, int]]:
    n = len(slots)
    inp = (Slot * max(1, n))()
    for i, t in enumerate(slots):
        inp[i] = Slot(*t)
    out = (S.StageSubOp * max(1, n))()
    cnt = C.c_int()
    rc = _lib().crosspipe_stage_ops(inp, n, stage, out, n, C.byref(cnt))
    if rc:
        raise RuntimeError(f"crosspipe_stage_ops failed ({rc})")
    return [(out[i].kind, out[i].mb, out[i].sub) for i in range(cnt.value)]
