"""The C++ scheduler core (sgprs_sched_*) against the Python oracle, on the CPU: both are driven
through the same seeded periodic task sets with a simulated clock and must take identical
decisions (which stage starts when, on which context and lane, at which level, with which
deadline) and count the same misses."""
import numpy as np
import pytest

import paper_2406_09425_amd as S
from oracle import sched_oracle as so


def run_core(n_contexts, lanes, tasks, horizon, exec_scale=1.0, offsets=None):
    """Event loop around the library: completions, then releases, then dispatches at each instant
    (the order the oracle's simulate() documents); release k of task i at offsets[i] + k * period."""
    sch = S.Sched(n_contexts, lanes)
    for (wcet, period, D) in tasks:
        sch.add_task(wcet, period, D)
    offsets = offsets or [0.0] * len(tasks)
    released = [0] * len(tasks)
    running = []   # [finish, order, task, job, stage]
    order = 0
    log = []
    while True:
        nxt = [offsets[i] + released[i] * tasks[i][1] for i in range(len(tasks))]
        times = [r[0] for r in running] + [t for t in nxt if t < horizon]
        if not times:
            break
        now = min(times)
        for ev in sorted(r for r in running if r[0] == now):
            running.remove(ev)
            sch.complete(ev[2], ev[3], ev[4], now)
        for i in range(len(tasks)):
            if nxt[i] < horizon and nxt[i] == now:
                assert sch.release(i, now) == released[i]
                released[i] += 1
        while True:
            d = sch.next(now)
            if d is None:
                break
            log.append((now, d.task, d.job, d.stage, d.context, d.lane, d.level, d.deadline))
            running.append([now + d.wcet * exec_scale, order, d.task, d.job, d.stage])
            order += 1
    st = sch.stats()
    sch.destroy()
    return log, st


def random_tasks(rng, n, n_stages, load):
    tasks = []
    for _ in range(n):
        wcet = [float(x) for x in np.round(rng.uniform(0.05, 0.6, n_stages), 3)]
        period = float(np.round(sum(wcet) * rng.uniform(1.5, 4.0) / load, 3))
        tasks.append((wcet, period, period * float(rng.choice([0.5, 1.0, 1.0]))))
    return tasks


@pytest.mark.parametrize("seed,n_ctx,lanes,n_tasks,n_stages,load,scale", [
    (0, 1, 1, 2, 3, 0.5, 1.0),      # one shared lane
    (1, 2, 2, 5, 6, 1.0, 1.0),
    (2, 3, 4, 9, 6, 2.0, 1.2),      # the paper's shape: 4 lanes, six stages, overloaded
    (3, 2, 4, 12, 6, 4.0, 1.5),     # far past the pivot point: misses, medium level, rule 3 of the assignment
    (4, 4, 3, 7, 2, 1.5, 0.8),      # odd lane count: one high lane, two low
    (5, 2, 8, 6, 10, 1.0, 1.0),
])
def test_core_takes_the_oracles_decisions(seed, n_ctx, lanes, n_tasks, n_stages, load, scale):
    rng = np.random.default_rng(seed)
    tasks = random_tasks(rng, n_tasks, n_stages, load)
    offsets = [float(x) for x in np.round(rng.uniform(0, 1.0, n_tasks), 3)]
    horizon = 12.0 * max(t[1] for t in tasks)
    ref_log, ref_st = so.simulate(n_ctx, lanes, tasks, horizon, scale, offsets)
    log, st = run_core(n_ctx, lanes, tasks, horizon, scale, offsets)
    assert len(ref_log) > 20 * n_tasks
    assert log == ref_log          # times, ids, contexts, lanes, levels and deadlines, bit for bit
    assert st == ref_st
    if load >= 2.0:
        assert st["stages_missed"] > 0 and any(e[6] == so.MEDIUM for e in log)


def test_offline_phase_matches_the_closed_form():
    sch = S.Sched(2, 4)
    t = sch.add_task([1.0, 2.0, 3.0], 12.0, 12.0)
    assert sch.virtual_deadlines(t, 3) == [2.0, 4.0, 6.0]
    w = [0.37, 1.9, 0.05, 0.6, 0.21, 0.9]
    t = sch.add_task(w, 33.3, 20.0)
    assert sch.virtual_deadlines(t, 6) == so.virtual_deadlines(w, 20.0)
    sch.destroy()


def test_paper_shape_hand_case():
    """One task of two stages on one context with a high and a low lane (the hand-worked case of
    the oracle's pins)."""
    log, st = run_core(1, 2, [([1.0, 1.0], 4.0, 4.0)], horizon=8.0)
    assert log == [(0.0, 0, 0, 0, 0, 1, 2, 2.0), (1.0, 0, 0, 1, 0, 0, 0, 4.0),
                   (4.0, 0, 1, 0, 0, 1, 2, 6.0), (5.0, 0, 1, 1, 0, 0, 0, 8.0)]
    assert st == dict(jobs_released=2, jobs_completed=2, jobs_missed=0, stages_completed=4, stages_missed=0)


def test_error_paths():
    with pytest.raises(S.SgprsError):
        S.Sched(0, 4)
    with pytest.raises(S.SgprsError):
        S.Sched(2, 9)
    sch = S.Sched(1, 2)
    with pytest.raises(S.SgprsError):
        sch.add_task([1.0, 0.0], 1.0, 1.0)     # a WCET of zero
    with pytest.raises(S.SgprsError):
        sch.add_task([1.0], 0.0, 1.0)
    with pytest.raises(S.SgprsError):
        sch.release(0, 0.0)                    # no such task
    t = sch.add_task([1.0, 1.0], 4.0, 4.0)
    with pytest.raises(S.SgprsError):
        sch.complete(t, 0, 0, 1.0)             # nothing is running
    sch.release(t, 0.0)
    assert sch.next(0.0) is not None and sch.next(0.0) is None
    with pytest.raises(S.SgprsError):
        sch.complete(t, 0, 1, 1.0)             # stage 1 has not started
    assert sch.complete(t, 0, 0, 2.5) is True  # after its deadline of 2.0
    d = sch.next(2.5)
    assert (d.stage, d.level, d.lane) == (1, 0, 0)
    sch.destroy()
