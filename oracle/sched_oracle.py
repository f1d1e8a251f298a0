"""CPU oracle for the CrossUDSub greedy schedule generator and the pipeline
performance model.

TEST INFRASTRUCTURE ONLY: the tests compare the library's host-side
generator / simulator (include/crosspipe_sched.h) with this file; nothing in
the product path imports it.

What it follows: the paper's Algorithm 1 ("Greedy Generation for CrossUDSub
Schedule") with the three steps of its scheduling loop (section 4.2.2: stage
selection, operation selection, operation scheduling), the range-based
bandwidth occupancy model (section 4.2.3), the alpha-beta communication model
(section 2.2) and the performance model of section 3.5 (start of a block =
max(end of the previous block on its stage, end of the block it depends on +
communication delay)).  The paper states the heuristic in prose only; the
readings taken here:

  * unidirectional pipeline, one model chunk per stage, stage == device;
    F(s,m) depends on F(s-1,m); D(s,m) on D(s+1,m) (on F(s,m) for the last
    stage); W(s,m) on D(s,m).  A dependent block becomes schedulable when the
    LAST sub-block of its predecessor has been scheduled (Alg. 1).
  * every block is cut into n_sub equal sub-blocks (duration T/n_sub).
  * memory: starting an F block adds M_F, finishing a D block adds M_D,
    finishing a W block adds M_W (M_W < 0 releases); an F block may start only
    if memory + M_F <= M_L.  D and W are never blocked by memory.
  * stage selection: the stage whose schedulable time
    max(end of its last scheduled sub-block, earliest T_avail of its feasible
    schedulable ops) is smallest; ties go to the lowest stage.
  * operation selection at that time t: only ops with T_avail <= t compete.
    A started, unfinished F or D block continues first (F and D stay whole);
    otherwise the stage's phase decides: warm-up is the time before the
    stage's first D arrives, when only F (within memory) and nothing else can
    run; from then on (steady) full blocks alternate -- after an F block prefer
    D, after a D block prefer F -- then the other type, then W; tear-down
    (every F of the stage scheduled) D > W.  Within a type the lowest
    microbatch goes first.  W advances one sub-block at a time.
  * communication starts when the producing block ends: it takes the earliest
    free window of length T_bw = beta * msg_bytes on the directed link at or
    after that time, and the consumer may start at window end + alpha.

Pins (tests/test_sched_pins.py): every dependency and the memory limit hold on
the produced timeline; 3*n_mb*n_sub*n_PP loop iterations; the simulator
reproduces the generator's own timeline; with no communication cost and the
memory of 1F1B the makespan equals the zero-bubble ZB-H1 closed form
n_mb*(T_F+T_D+T_W) + (n_PP-1)*(T_F+T_D-T_W); a hand-worked 2-stage example;
monotonicity in the memory limit and in the delays.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

F, D, W = 0, 1, 2


@dataclass
class Params:
    n_pp: int
    n_mb: int
    n_sub: int
    t_f: Sequence[float]          # per stage, full-block durations
    t_d: Sequence[float]
    t_w: Sequence[float]
    m_f: float = 1.0              # net memory change of a full F / D / W block
    m_d: float = 0.0
    m_w: float = -1.0
    m_limit: float = 1e30         # per-stage memory limit M_L
    alpha: Sequence[Sequence[float]] = None   # [i][j] latency device i -> j
    beta: Sequence[Sequence[float]] = None    # [i][j] inverse bandwidth (time per byte)
    msg_bytes: float = 0.0

    def dur(self, stage, kind):
        return (self.t_f, self.t_d, self.t_w)[kind][stage] / self.n_sub


@dataclass
class Slot:
    stage: int
    kind: int
    mb: int
    sub: int
    t_start: float
    t_end: float


class Link:
    """Occupied transmission windows of one directed link (section 4.2.3)."""

    def __init__(self):
        self.busy: List[Tuple[float, float]] = []

    def reserve(self, t_ready: float, t_bw: float) -> float:
        """Earliest window of length t_bw starting at or after t_ready; returns its end."""
        if t_bw <= 0.0:
            return t_ready
        start = t_ready
        for a, b in self.busy:                       # sorted by start
            if start + t_bw <= a:
                break
            if b > start:
                start = b
        self.busy.append((start, start + t_bw))
        self.busy.sort()
        return start + t_bw


def _comm(p: Params, links, src: int, dst: int, t_ready: float) -> float:
    a = p.alpha[src][dst] if p.alpha is not None else 0.0
    b = p.beta[src][dst] if p.beta is not None else 0.0
    return links[(src, dst)].reserve(t_ready, b * p.msg_bytes) + a


def _successor(p: Params, stage: int, kind: int):
    """(stage, kind) of the block that depends on a finished (stage, kind) block across stages, or None."""
    if kind == F:
        return (stage + 1, F) if stage + 1 < p.n_pp else (stage, D)
    if kind == D:
        return (stage - 1, D) if stage > 0 else None
    return None


@dataclass
class _StageState:
    end: float = 0.0
    mem: float = 0.0
    avail: dict = field(default_factory=dict)        # (kind, mb) -> T_avail of schedulable blocks
    done_sub: dict = field(default_factory=dict)     # (kind, mb) -> sub-blocks already scheduled
    n_f_started: int = 0
    n_d_started: int = 0
    last_full: int = -1                              # kind of the last F/D block started


def greedy(p: Params):
    """Returns (slots in scheduling order, makespan, loop iterations)."""
    st = [_StageState() for _ in range(p.n_pp)]
    links = {(i, j): Link() for i in range(p.n_pp) for j in range(p.n_pp) if i != j}
    for m in range(p.n_mb):
        st[0].avail[(F, m)] = 0.0
    slots: List[Slot] = []
    iters = 0
    while True:
        # --- stage selection
        best = None
        for s in range(p.n_pp):
            cands = _feasible(p, st[s])
            if not cands:
                continue
            t = max(st[s].end, min(st[s].avail[c] for c in cands))
            if best is None or t < best[0]:
                best = (t, s)
        if best is None:
            break
        t, s = best
        S = st[s]
        # --- operation selection
        kind, mb = _select(p, S, [c for c in _feasible(p, S) if S.avail[c] <= t])
        # --- operation scheduling
        sub = S.done_sub.get((kind, mb), 0)
        sub_idx = p.n_sub - 1 - sub if kind == D else sub       # D walks the layer groups backwards
        if sub == 0:
            if kind == F:
                S.mem += p.m_f; S.n_f_started += 1; S.last_full = F
            elif kind == D:
                S.n_d_started += 1; S.last_full = D
        t_end = t + p.dur(s, kind)
        slots.append(Slot(s, kind, mb, sub_idx, t, t_end))
        S.end = t_end
        S.done_sub[(kind, mb)] = sub + 1
        iters += 1
        if sub + 1 == p.n_sub:                                    # block complete
            del S.avail[(kind, mb)]
            if kind == D:
                S.mem += p.m_d
                S.avail[(W, mb)] = t_end
            elif kind == W:
                S.mem += p.m_w
            nxt = _successor(p, s, kind)
            if nxt is not None:
                ns, nk = nxt
                st[ns].avail[(nk, mb)] = t_end if ns == s else _comm(p, links, s, ns, t_end)
    return slots, max((x.t_end for x in slots), default=0.0), iters


def _feasible(p: Params, S: _StageState):
    out = []
    for (kind, mb) in S.avail:
        if kind == F and S.done_sub.get((kind, mb), 0) == 0 and S.mem + p.m_f > p.m_limit + 1e-12:
            continue                                              # memory prevents starting this F block
        out.append((kind, mb))
    return out


def _select(p: Params, S: _StageState, cands):
    started = [c for c in cands if c[0] != W and 0 < S.done_sub.get(c, 0) < p.n_sub]
    if started:
        return min(started, key=lambda c: (c[0], c[1]))
    by = {k: sorted(m for (kk, m) in cands if kk == k) for k in (F, D, W)}
    if S.n_f_started >= p.n_mb:
        order = (D, W)                                            # tear-down
    else:                                                         # warm-up (no D has arrived yet: F) / steady (alternate)
        order = (F, D, W) if S.last_full == D else (D, F, W)
    for k in order:
        if by[k]:
            return k, by[k][0]
    return W, by[W][0]


def simulate(p: Params, per_stage: List[List[Tuple[int, int, int]]]):
    """Performance model (section 3.5): per_stage[s] = ordered (kind, mb, sub) list of stage s.
    Returns (timed slots, makespan); raises ValueError on a list that can never complete."""
    pos = [0] * p.n_pp
    end = [0.0] * p.n_pp
    links = {(i, j): Link() for i in range(p.n_pp) for j in range(p.n_pp) if i != j}
    avail = [dict() for _ in range(p.n_pp)]                        # (kind, mb) -> time its input arrives
    done = [dict() for _ in range(p.n_pp)]
    for m in range(p.n_mb):
        avail[0][(F, m)] = 0.0
    out: List[Slot] = []
    total = sum(len(l) for l in per_stage)
    while len(out) < total:
        best = None
        for s in range(p.n_pp):
            if pos[s] >= len(per_stage[s]):
                continue
            kind, mb, sub = per_stage[s][pos[s]]
            if (kind, mb) not in avail[s]:
                continue
            t = max(end[s], avail[s][(kind, mb)])
            if best is None or t < best[0]:
                best = (t, s)
        if best is None:
            raise ValueError("schedule deadlocks: no stage can run its next op")
        t, s = best
        kind, mb, sub = per_stage[s][pos[s]]
        pos[s] += 1
        t_end = t + p.dur(s, kind)
        out.append(Slot(s, kind, mb, sub, t, t_end))
        end[s] = t_end
        done[s][(kind, mb)] = done[s].get((kind, mb), 0) + 1
        if done[s][(kind, mb)] == p.n_sub:
            if kind == D:
                avail[s][(W, mb)] = t_end
            nxt = _successor(p, s, kind)
            if nxt is not None:
                ns, nk = nxt
                avail[ns][(nk, mb)] = t_end if ns == s else _comm(p, links, s, ns, t_end)
    return out, max((x.t_end for x in out), default=0.0)


def per_stage_lists(p: Params, slots: List[Slot]):
    lists = [[] for _ in range(p.n_pp)]
    for x in slots:
        lists[x.stage].append((x.kind, x.mb, x.sub))
    return lists
