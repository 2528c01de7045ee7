"""CPU tests of the pipeline schedule simulator: the paper's worked example and the
invariants every valid schedule has."""
import itertools
import os

import pytest

from paper_2111_04007_amd import schedule_sim as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "schedule_worked_example.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = [p.strip() for p in line.split("=")]
            out[k] = float(v)
    return out


def test_paper_worked_example():
    g = _golden()
    P, N = int(g["stages"]), int(g["micro_batches"])
    v = S.simulate("varuna", P, N, g["forward"], g["backward"], g["recompute"])
    p = S.simulate("gpipe", P, N, g["forward"], g["backward"], g["recompute"])
    assert p.makespan - v.makespan == g["gpipe_minus_varuna"]
    assert v.count(P - 1, "R") == g["varuna_last_stage_recomputes"]
    assert p.count(P - 1, "R") == g["gpipe_last_stage_recomputes"]
    # the one recompute GPipe's last stage avoids is the fifth micro-batch's
    assert sorted(t.mb for t in p.stage_tasks(P - 1) if t.kind == "R") == [0, 1, 2, 3]
    # every other stage recomputes every micro-batch in both schedules
    for s in range(P - 1):
        assert v.count(s, "R") == N and p.count(s, "R") == N


def _check_valid(res, P, N, F, B, R, send):
    by = {(t.stage, t.kind, t.mb): t for t in res.tasks}
    for s in range(P):
        ts = res.stage_tasks(s)
        assert sum(1 for t in ts if t.kind == "F") == N and sum(1 for t in ts if t.kind == "B") == N
        for a, b in zip(ts, ts[1:]):
            assert b.start >= a.end - 1e-12, "a stage runs one task at a time"
        for mb in range(N):
            f, b = by[(s, "F", mb)], by[(s, "B", mb)]
            assert abs((f.end - f.start) - F[s]) < 1e-12 and abs((b.end - b.start) - B[s]) < 1e-12
            if s > 0:
                assert f.start >= by[(s - 1, "F", mb)].end + send - 1e-12
            if s < P - 1:
                assert b.start >= by[(s + 1, "B", mb)].end + send - 1e-12
            else:
                assert b.start >= f.end - 1e-12
            r = by.get((s, "R", mb))
            if r is not None:
                assert f.end <= r.start + 1e-12 and r.end <= b.start + 1e-12
                assert abs((r.end - r.start) - R[s]) < 1e-12
                if res.schedule == "varuna":   # rule 2: nothing between a recompute and its backward
                    i = ts.index(r)
                    assert ts[i + 1] is b
            else:
                # only a backward that directly follows its own forward may skip the recompute
                i = ts.index(f)
                assert ts[i + 1] is b


@pytest.mark.parametrize("P,N", list(itertools.product([1, 2, 3, 4, 6, 9], [1, 2, 5, 8, 17])))
def test_schedules_are_valid_and_varuna_is_no_slower(P, N):
    F, B, R = [1.0] * P, [2.0] * P, [1.0] * P
    v = S.simulate("varuna", P, N, 1.0, 2.0)
    g = S.simulate("gpipe", P, N, 1.0, 2.0)
    _check_valid(v, P, N, F, B, R, 0.0)
    _check_valid(g, P, N, F, B, R, 0.0)
    assert v.makespan <= g.makespan
    # lower bounds: the busiest stage's work; the critical path of the first micro-batch
    work = N * (4.0 if P > 1 else 3.0)
    assert v.makespan >= work - 1e-12 and g.makespan >= work - 1e-12
    assert v.makespan >= P * 1.0 + P * 2.0 - 1e-12


def test_single_stage_and_nonuniform_stages_with_latency():
    r = S.simulate("varuna", 1, 7, 1.5, 2.5)
    assert r.makespan == 7 * 4.0 and r.count(0, "R") == 0
    F, B, R = [1.0, 1.3, 0.7], [2.2, 2.0, 1.9], [0.9, 1.3, 0.7]
    for sch in ("varuna", "gpipe"):
        res = S.simulate(sch, 3, 6, F, B, R, send=0.25, allreduce=3.0)
        _check_valid(res, 3, 6, F, B, R, 0.25)
        assert res.minibatch_time == res.makespan + 3.0
    with pytest.raises(ValueError):
        S.simulate("1f1b", 2, 2, 1, 2)
    with pytest.raises(ValueError):
        S.simulate("varuna", 3, 2, [1, 2], 2)


def test_estimate_from_measured_stage_times():
    """Fed with stage times of the shape this library measures (ms): more micro-batches
    amortise the pipeline fill, and the estimate is bounded below by one stage's work."""
    e8 = S.estimate(4, 8, f_ms=5.8, rb_ms=19.7, f_last_ms=6.0, b_last_ms=15.2, allreduce_ms=40.0)
    e64 = S.estimate(4, 64, f_ms=5.8, rb_ms=19.7, f_last_ms=6.0, b_last_ms=15.2, allreduce_ms=40.0)
    for e, n in ((e8, 8), (e64, 64)):
        for sch in ("varuna", "gpipe"):
            assert e[sch + "_ms"] >= n * (5.8 + 19.7) + 40.0          # one middle stage's work + all-reduce
            assert 0.0 < e[sch + "_bubble_frac"] < 0.5
    assert e64["varuna_bubble_frac"] < e8["varuna_bubble_frac"]
    assert e64["gpipe_bubble_frac"] < e8["gpipe_bubble_frac"]
