"""Pins for the scheduler oracle (oracle/sched_oracle.py): values worked out by hand from the
paper's rules ("Offline Phase", "Online Phase").  The paper prints no worked example of the
scheduler, so the pins are the closed forms and small cases its rules fix; each one is chosen so
that a plausible slip (wrong proportion, cumulative vs. per-stage deadline, wrong tie order,
wrong lane class, medium level forgotten) fails it."""
import pytest

from oracle import sched_oracle as so

HIGH, MEDIUM, LOW = so.HIGH, so.MEDIUM, so.LOW


def test_virtual_deadlines_are_wcet_proportional():
    # "WCET and Virtual Deadline Assignment": C = (1, 2, 3), D = 12 -> (2, 4, 6)
    assert so.virtual_deadlines([1.0, 2.0, 3.0], 12.0) == [2.0, 4.0, 6.0]
    v = so.virtual_deadlines([0.3, 1.7, 0.25, 4.0], 33.3)
    assert abs(sum(v) - 33.3) < 1e-12
    assert abs(v[1] / v[0] - 1.7 / 0.3) < 1e-12 and abs(v[3] / v[2] - 16.0) < 1e-12


def test_two_level_priority_and_medium_level():
    # last stage high, the others low; a low stage after a missed one becomes medium
    assert [so.stage_level(j, 6, False) for j in range(6)] == [LOW] * 5 + [HIGH]
    assert so.stage_level(2, 6, True) == MEDIUM
    assert so.stage_level(5, 6, True) == HIGH  # the last stage stays high
    assert HIGH < MEDIUM < LOW


def test_absolute_deadlines_accumulate_to_the_job_deadline():
    vdl = [2.0, 4.0, 6.0]
    assert [so.absolute_deadline(10.0, vdl, j) for j in range(3)] == [12.0, 16.0, 22.0]


def _stage(wcet, deadline, level=LOW, seq=0, start=None):
    d = dict(task=0, job=seq, stage=0, level=level, wcet=wcet, deadline=deadline, seq=seq)
    if start is not None:
        d["start"] = start
    return d


def test_context_assignment_three_rules():
    s = so.Scheduler(2, 4)
    s.waiting[0].append(_stage(1.0, 9.0))
    assert s.assign_context(0.0, 1.0, 5.0) == 1            # an empty queue first
    # context 0: two stages, backlog 5; context 1: one stage, backlog 8
    s = so.Scheduler(2, 4)
    s.waiting[0] += [_stage(2.0, 50.0, seq=0), _stage(3.0, 50.0, seq=1)]
    s.waiting[1] += [_stage(8.0, 50.0, seq=2)]
    now = 100.0
    assert s.assign_context(now, 1.0, now + 20.0) == 1     # both meet it: the shorter queue
    assert s.assign_context(now, 1.0, now + 7.0) == 0      # only context 0 meets it (5 + 1 <= 7)
    assert s.assign_context(now, 1.0, now + 3.0) == 0      # none does: the earlier finish (5 < 8)
    # running stages count with what is left of them: 8 - (100 - 95) = 3 < 5
    s.waiting[1].clear()
    s.running[1][2] = _stage(8.0, 50.0, seq=2, start=95.0)
    assert s.backlog(1, now) == 3.0
    assert s.assign_context(now, 1.0, now + 3.0) == 1
    # equal queues and both meeting: the lower index
    s = so.Scheduler(3, 2)
    for c in range(3):
        s.waiting[c].append(_stage(1.0, 50.0, seq=c))
    assert s.assign_context(0.0, 1.0, 10.0) == 0


def test_lane_classes_and_edf_inside_a_level():
    s = so.Scheduler(1, 4)
    s.waiting[0] += [_stage(1, 5.0, LOW, 0), _stage(1, 9.0, MEDIUM, 1), _stage(1, 20.0, HIGH, 2), _stage(1, 3.0, LOW, 3),
                     _stage(1, 4.0, MEDIUM, 4)]
    got = []
    while True:
        d = s.next(0.0)
        if d is None:
            break
        got.append((d["lane"], d["level"], d["deadline"]))
    # lane 0 (high) takes the high stage, lane 1 (high) stays empty, lanes 2 and 3 (low) take the
    # medium stages in deadline order before any low one
    assert got == [(0, HIGH, 20.0), (2, MEDIUM, 4.0), (3, MEDIUM, 9.0)]
    assert [x["deadline"] for x in s.waiting[0]] == [5.0, 3.0]
    # a single lane is shared by every level: high, then medium, then low by deadline
    s = so.Scheduler(1, 1)
    s.waiting[0] += [_stage(1, 5.0, LOW, 0), _stage(1, 20.0, HIGH, 1), _stage(1, 3.0, LOW, 2), _stage(1, 9.0, MEDIUM, 3)]
    order = []
    for _ in range(4):
        d = s.next(0.0)
        order.append((d["level"], d["deadline"]))
        s.running[0][0] = None
    assert order == [(HIGH, 20.0), (MEDIUM, 9.0), (LOW, 3.0), (LOW, 5.0)]


def test_equal_deadlines_go_in_release_order():
    s = so.Scheduler(1, 1)
    s.waiting[0] += [_stage(1, 5.0, LOW, 7), _stage(1, 5.0, LOW, 3)]
    assert s.next(0.0)["seq"] == 3


def test_hand_simulation_without_misses():
    # one task, C = (1, 1), T = D = 4, one context with a high and a low lane
    log, st = so.simulate(1, 2, [([1.0, 1.0], 4.0, 4.0)], horizon=8.0)
    assert log == [(0.0, 0, 0, 0, 0, 1, LOW, 2.0), (1.0, 0, 0, 1, 0, 0, HIGH, 4.0),
                   (4.0, 0, 1, 0, 0, 1, LOW, 6.0), (5.0, 0, 1, 1, 0, 0, HIGH, 8.0)]
    assert st == dict(jobs_released=2, jobs_completed=2, jobs_missed=0, stages_completed=4, stages_missed=0)


def test_hand_simulation_with_misses_and_medium_promotion():
    # one context, one lane; C = (2, 1, 1), T = 5, D = 4 -> virtual deadlines (2, 1, 1);
    # the stages take twice their WCET.
    # job 0 (r = 0): stage 0 runs 0-4, d = 2: missed -> stage 1 is medium, d = 3, runs 4-6: missed ->
    # stage 2 is high, d = 4, runs 6-8: job missed.  Job 1 (r = 5): stage 0 low, d = 7, waits for the
    # lane until 8 (the high stage of job 0 was released at 6 and goes first), runs 8-12: missed ...
    log, st = so.simulate(1, 1, [([2.0, 1.0, 1.0], 5.0, 4.0)], horizon=6.0, exec_scale=2.0)
    assert log == [(0.0, 0, 0, 0, 0, 0, LOW, 2.0), (4.0, 0, 0, 1, 0, 0, MEDIUM, 3.0), (6.0, 0, 0, 2, 0, 0, HIGH, 4.0),
                   (8.0, 0, 1, 0, 0, 0, LOW, 7.0), (12.0, 0, 1, 1, 0, 0, MEDIUM, 8.0), (14.0, 0, 1, 2, 0, 0, HIGH, 9.0)]
    assert st == dict(jobs_released=2, jobs_completed=2, jobs_missed=2, stages_completed=6, stages_missed=6)


def test_a_stage_finishing_exactly_on_its_deadline_is_not_a_miss():
    log, st = so.simulate(1, 1, [([1.0, 1.0], 10.0, 2.0)], horizon=1.0)
    assert st["stages_missed"] == 0 and st["jobs_missed"] == 0


def test_two_contexts_spread_simultaneous_releases():
    # three identical tasks released together on two contexts: the first two find empty queues,
    # the third meets its deadline on either and takes the lower index among equal queue lengths
    tasks = [([1.0, 1.0], 100.0, 100.0)] * 3
    log, _ = so.simulate(2, 2, tasks, horizon=1.0)
    first = [(e[1], e[4]) for e in log if e[3] == 0]
    assert sorted(first) == [(0, 0), (1, 1), (2, 0)]


def test_invariants_on_a_loaded_system():
    tasks = [([0.4, 0.3, 0.2, 0.5, 0.3, 0.1], 3.3, 3.3)] * 9
    log, st = so.simulate(3, 4, tasks, horizon=40.0, exec_scale=1.3, offsets=[0.1 * i for i in range(9)])
    assert st["jobs_completed"] == st["jobs_released"] and st["stages_completed"] == 6 * st["jobs_completed"]
    starts = {}
    for (t, task, job, stage, ctx, lane, level, dl) in log:
        assert (task, job, stage) not in starts
        starts[(task, job, stage)] = t
        if stage:   # precedence inside a job
            assert starts[(task, job, stage - 1)] + tasks[task][0][stage - 1] * 1.3 <= t + 1e-12
        assert (level == HIGH) == (stage == 5)
        assert (lane < 2) == (level == HIGH)   # lane classes
    # a lane never runs two stages at once
    busy = {}
    for (t, task, job, stage, ctx, lane, level, dl) in log:
        assert busy.get((ctx, lane), -1.0) <= t + 1e-12
        busy[(ctx, lane)] = t + tasks[task][0][stage] * 1.3
