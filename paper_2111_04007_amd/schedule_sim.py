"""Event-driven simulation of one mini-batch on a P-stage pipeline (CPU only).

Feeds on the per-stage compute times this library measures (forward F, recompute R,
backward B per micro-batch; `calibrate.sweep`) and estimates the time of a mini-batch of
N_m micro-batches followed by the gradient all-reduce, as the paper's morphing does
(Job Morphing, "Parametrized Simulation").  Two schedules:

* ``varuna``: the paper's rule-based schedule (Design Overview, "Tuning pipeline
  efficiency").  Rule 1: the recompute of micro-batch m on stage k-1 is placed so that it
  ends when the gradient of m arrives from stage k, i.e. it may start once stage k has
  begun that backward pass (backward takes longer than a forward).  Rule 2: after a
  recompute the stage runs nothing but the matching backward.  Rule 3: with both a forward
  and a backward ready, the backward goes first.  The last stage runs each backward
  straight after its forward and never recomputes.
* ``gpipe``: all forwards, then backwards in reverse micro-batch order, each preceded by a
  recompute (the last stage skips it only for the micro-batch it has just forwarded).

Times are in any one unit; `send` is the latency of handing an activation or a gradient to
the neighbouring stage.  The simulation is deterministic and work-conserving within the
rules.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple


@dataclass
class Task:
    stage: int
    kind: str        # "F", "R" or "B"
    mb: int
    start: float
    end: float


@dataclass
class Result:
    schedule: str
    makespan: float                       # pipeline part: first forward start to last backward end
    minibatch_time: float                 # makespan + allreduce
    tasks: List[Task] = field(default_factory=list)

    def stage_tasks(self, stage: int) -> List[Task]:
        return sorted((t for t in self.tasks if t.stage == stage), key=lambda t: t.start)

    def count(self, stage: int, kind: str) -> int:
        return sum(1 for t in self.tasks if t.stage == stage and t.kind == kind)

    def busy(self, stage: int) -> float:
        return sum(t.end - t.start for t in self.tasks if t.stage == stage)

    def timeline(self, unit: float = 1.0) -> str:
        """One text row per stage, one column per `unit` of time (for uniform integer times)."""
        n = int(round(self.makespan / unit))
        rows = []
        for s in range(1 + max(t.stage for t in self.tasks)):
            cells = ["  . "] * n
            for t in self.stage_tasks(s):
                for c in range(int(round(t.start / unit)), int(round(t.end / unit))):
                    cells[c] = f"{t.kind}{t.mb + 1:<3d}"
            rows.append(f"S{s + 1} " + "".join(cells))
        return "\n".join(rows)


def _per_stage(x, n_stages: int) -> List[float]:
    if isinstance(x, (int, float)):
        return [float(x)] * n_stages
    x = [float(v) for v in x]
    if len(x) != n_stages:
        raise ValueError(f"expected {n_stages} per-stage times, got {len(x)}")
    return x


def simulate(schedule: str, n_stages: int, n_micro_batches: int, forward, backward, recompute=None,
             send: float = 0.0, allreduce: float = 0.0) -> Result:
    """Simulates one mini-batch.  forward / backward / recompute: a number (uniform stages) or
    one value per stage; recompute defaults to forward."""
    if schedule not in ("varuna", "gpipe"):
        raise ValueError("schedule must be 'varuna' or 'gpipe'")
    if n_stages < 1 or n_micro_batches < 1:
        raise ValueError("need at least one stage and one micro-batch")
    P, N = n_stages, n_micro_batches
    F = _per_stage(forward, P)
    B = _per_stage(backward, P)
    R = _per_stage(F if recompute is None else recompute, P)
    last = P - 1
    INF = float("inf")

    act_ready = [[0.0 if s == 0 else INF for _ in range(N)] for s in range(P)]   # input activation of (s, mb)
    grad_ready = [[INF] * N for _ in range(P)]                                  # output gradient of (s, mb)
    b_started = [[INF] * N for _ in range(P)]                                   # start time of B(s, mb)
    fwd_done = [[False] * N for _ in range(P)]
    rec_done = [[False] * N for _ in range(P)]
    bwd_done = [[False] * N for _ in range(P)]
    free_at = [0.0] * P
    waiting_b = [-1] * P      # rule 2: micro-batch whose recompute is done and whose backward must come next
    tasks: List[Task] = []

    def run(s, kind, mb, t0):
        dur = {"F": F, "R": R, "B": B}[kind][s]
        t1 = t0 + dur
        tasks.append(Task(s, kind, mb, t0, t1))
        free_at[s] = t1
        if kind == "F":
            fwd_done[s][mb] = True
            if s < last:
                act_ready[s + 1][mb] = t1 + send
            else:
                grad_ready[s][mb] = t1      # the loss gradient is available as soon as the forward ends
        elif kind == "R":
            rec_done[s][mb] = True
            waiting_b[s] = mb
        else:
            bwd_done[s][mb] = True
            b_started[s][mb] = t0
            waiting_b[s] = -1
            if s > 0:
                grad_ready[s - 1][mb] = t1 + send

    def next_task(s, now):
        """(kind, mb, earliest start) of what stage s runs next, or None if it has to wait for an event."""
        # last stage: backward straight after forward, no recompute
        if s == last and schedule == "varuna" or (s == last and P == 1):
            for mb in range(N):
                if fwd_done[s][mb] and not bwd_done[s][mb]:
                    return ("B", mb, max(now, grad_ready[s][mb]))
            for mb in range(N):
                if not fwd_done[s][mb]:
                    return ("F", mb, max(now, act_ready[s][mb])) if act_ready[s][mb] < INF else None
            return None
        if schedule == "gpipe":
            for mb in range(N):                         # all forwards first, in order
                if not fwd_done[s][mb]:
                    return ("F", mb, max(now, act_ready[s][mb])) if act_ready[s][mb] < INF else None
            for mb in range(N - 1, -1, -1):             # then backwards, newest micro-batch first
                if bwd_done[s][mb]:
                    continue
                needs_r = not (s == last and mb == N - 1)   # activations of the last forward are still there
                if needs_r and not rec_done[s][mb]:
                    # recompute as late as it can be without delaying the backward
                    g = grad_ready[s][mb]
                    return ("R", mb, max(now, g - R[s])) if g < INF else None
                g = grad_ready[s][mb]
                return ("B", mb, max(now, g)) if g < INF else None
            return None
        # varuna, stages before the last
        if waiting_b[s] >= 0:                           # rule 2
            mb = waiting_b[s]
            g = grad_ready[s][mb]
            return ("B", mb, max(now, g)) if g < INF else None
        # rule 1: a recompute is placed just in time -- it ends when the gradient arrives from
        # the next stage, whose backward of that micro-batch must therefore have begun
        rec = None
        for mb in range(N):
            if fwd_done[s][mb] and not bwd_done[s][mb] and not rec_done[s][mb]:
                t0 = b_started[s + 1][mb]
                if t0 < INF:
                    r0 = max(now, t0 + B[s + 1] + send - R[s])
                    if rec is None or r0 < rec[0]:
                        rec = (r0, mb)
        fwd = None
        for mb in range(N):
            if not fwd_done[s][mb]:
                if act_ready[s][mb] < INF:
                    fwd = (max(now, act_ready[s][mb]), mb)
                break
        # rule 3: backward work first -- a forward runs only if it is over before the recompute is due
        if rec is not None and (fwd is None or fwd[0] + F[s] > rec[0] + 1e-12):
            return ("R", rec[1], rec[0])
        if fwd is not None:
            return ("F", fwd[1], fwd[0])
        return None

    # global event loop: repeatedly start the task that can start earliest
    total = sum(N * (3 if (s != last or schedule == "gpipe") else 2) for s in range(P))
    guard = 0
    while True:
        best = None
        for s in range(P):
            nt = next_task(s, free_at[s])
            if nt is not None and (best is None or (nt[2], s) < (best[1][2], best[0])):
                best = (s, nt)
        if best is None:
            break
        s, (kind, mb, t0) = best
        run(s, kind, mb, t0)
        guard += 1
        if guard > 4 * total + 16:
            raise RuntimeError("schedule simulation does not terminate")
    if not all(all(row) for row in bwd_done):
        raise RuntimeError("schedule simulation stalled before every backward ran")
    makespan = max(t.end for t in tasks)
    return Result(schedule, makespan, makespan + allreduce, tasks)


def estimate(n_stages: int, n_micro_batches: int, f_ms: float, rb_ms: float, f_last_ms: float, b_last_ms: float,
             r_ms: float = None, send_ms: float = 0.0, allreduce_ms: float = 0.0) -> Dict[str, float]:
    """Mini-batch time estimate from this library's measured stage times: middle stages take
    f_ms per forward and rb_ms per recompute+backward (split into r_ms, default f_ms, and the
    rest), the last stage f_last_ms and b_last_ms."""
    r = f_ms if r_ms is None else r_ms
    fw = [f_ms] * (n_stages - 1) + [f_last_ms]
    bw = [rb_ms - r] * (n_stages - 1) + [b_last_ms]
    rc = [r] * n_stages
    out = {}
    for sch in ("varuna", "gpipe"):
        res = simulate(sch, n_stages, n_micro_batches, fw, bw, rc, send_ms, allreduce_ms)
        out[sch + "_ms"] = res.minibatch_time
        out[sch + "_bubble_frac"] = 1.0 - sum(res.busy(s) for s in range(n_stages)) / (n_stages * res.makespan)
    return out
