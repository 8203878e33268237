"""Plain Python statement of the SGPRS scheduling rules (test infrastructure only).

Written from the paper's sections "Task Model", "Offline Phase" (Two Level Priority
Assignment, WCET and Virtual Deadline Assignment) and "Online Phase" (Absolute Deadline
Assignment, Context Assignment, Stage Queuing).  Lists and loops, nothing clever: a reader
checks it against the paper by eye.  Only tests may import this module; the product's
scheduler (C++) shares no code with it.

Readings taken where the paper is silent (each also listed in the design notes):
  * absolute deadline of stage j of a job released at r: d = r + D^0 + ... + D^j, so the
    last stage's deadline is the job's own (r + D);
  * a context's queue = its stages that are waiting or running; its backlog = the WCETs
    of the waiting ones plus what is left of the running ones; "meets the deadline" means
    now + backlog + C <= d; ties go to the lowest context index;
  * a context has `lanes` streams, the first lanes // 2 for high-priority stages and the
    rest for medium and low ones (the paper: two and two); with a single lane every stage
    shares it;
  * inside a level the earliest absolute deadline goes first, ties by order of release;
  * a deadline is missed when the stage completes strictly after it.
"""
from __future__ import annotations

HIGH, MEDIUM, LOW = 0, 1, 2


def virtual_deadlines(wcet, rel_deadline):
    """'WCET and Virtual Deadline Assignment': D^j = D * C^j / sum_k C^k."""
    total = 0.0
    for c in wcet:
        total += c
    return [rel_deadline * c / total for c in wcet]


def stage_level(stage, n_stages, previous_stage_missed):
    """'Two Level Priority Assignment' + the medium level of 'Stage Queuing'."""
    if stage == n_stages - 1:
        return HIGH
    return MEDIUM if previous_stage_missed else LOW


def absolute_deadline(job_release, vdl, stage):
    """'Absolute Deadline Assignment' (cumulative reading, see the module text)."""
    d = job_release
    for k in range(stage + 1):
        d += vdl[k]
    return d


class Scheduler:
    """The online phase: context assignment at release, per-lane choice at dispatch."""

    def __init__(self, n_contexts, lanes):
        self.n_contexts, self.lanes = n_contexts, lanes
        self.n_high = lanes // 2
        self.tasks = []          # dicts: wcet, vdl, period, D, jobs
        self.waiting = [[] for _ in range(n_contexts)]            # stage records
        self.running = [[None] * lanes for _ in range(n_contexts)]
        self.seq = 0
        self.stats = dict(jobs_released=0, jobs_completed=0, jobs_missed=0, stages_completed=0, stages_missed=0)
        self.jobs = {}

    # ---- offline phase
    def add_task(self, wcet, period, rel_deadline):
        self.tasks.append(dict(wcet=list(wcet), vdl=virtual_deadlines(wcet, rel_deadline), period=period,
                               D=rel_deadline, next_job=0))
        return len(self.tasks) - 1

    # ---- online phase
    def backlog(self, c, now):
        b = 0.0
        for s in self.waiting[c]:
            b += s["wcet"]
        for s in self.running[c]:
            if s is not None:
                b += max(0.0, s["wcet"] - (now - s["start"]))
        return b

    def queue_len(self, c):
        return len(self.waiting[c]) + sum(1 for s in self.running[c] if s is not None)

    def assign_context(self, now, wcet, deadline):
        """'Context Assignment': empty queue, else shortest queue among those that meet the
        deadline, else earliest finish."""
        for c in range(self.n_contexts):
            if self.queue_len(c) == 0:
                return c
        best = None
        for c in range(self.n_contexts):
            if now + self.backlog(c, now) + wcet <= deadline:
                if best is None or self.queue_len(c) < self.queue_len(best):
                    best = c
        if best is not None:
            return best
        for c in range(self.n_contexts):
            if best is None or now + self.backlog(c, now) < now + self.backlog(best, now):
                best = c
        return best

    def _release_stage(self, task, job, stage, now):
        t = self.tasks[task]
        j = self.jobs[(task, job)]
        rec = dict(task=task, job=job, stage=stage, level=stage_level(stage, len(t["wcet"]), j["prev_missed"]),
                   wcet=t["wcet"][stage], deadline=absolute_deadline(j["release"], t["vdl"], stage), seq=self.seq)
        self.seq += 1
        rec["context"] = self.assign_context(now, rec["wcet"], rec["deadline"])
        self.waiting[rec["context"]].append(rec)

    def release(self, task, now):
        t = self.tasks[task]
        job = t["next_job"]
        t["next_job"] += 1
        self.jobs[(task, job)] = dict(release=now, prev_missed=False)
        self.stats["jobs_released"] += 1
        self._release_stage(task, job, 0, now)
        return job

    def next(self, now):
        """One stage that may start now, or None ('Stage Queuing')."""
        for c in range(self.n_contexts):
            for lane in range(self.lanes):
                if self.running[c][lane] is not None:
                    continue
                best = None
                for s in self.waiting[c]:
                    if self.lanes > 1:
                        if lane < self.n_high and s["level"] != HIGH:
                            continue
                        if lane >= self.n_high and s["level"] == HIGH:
                            continue
                    key = (s["level"], s["deadline"], s["seq"])
                    if best is None or key < (best["level"], best["deadline"], best["seq"]):
                        best = s
                if best is not None:
                    self.waiting[c].remove(best)
                    best["lane"], best["start"] = lane, now
                    self.running[c][lane] = best
                    return best
        return None

    def complete(self, task, job, stage, now):
        for c in range(self.n_contexts):
            for lane in range(self.lanes):
                s = self.running[c][lane]
                if s is not None and (s["task"], s["job"], s["stage"]) == (task, job, stage):
                    self.running[c][lane] = None
                    missed = now > s["deadline"]
                    self.stats["stages_completed"] += 1
                    self.stats["stages_missed"] += int(missed)
                    n_stages = len(self.tasks[task]["wcet"])
                    if stage + 1 < n_stages:
                        self.jobs[(task, job)]["prev_missed"] = missed
                        self._release_stage(task, job, stage + 1, now)
                    else:
                        self.stats["jobs_completed"] += 1
                        self.stats["jobs_missed"] += int(missed)
                        del self.jobs[(task, job)]
                    return missed
        raise KeyError((task, job, stage))


def simulate(n_contexts, lanes, tasks, horizon, exec_scale=1.0, offsets=None):
    """Discrete-event run: task i releases a job at offsets[i] + k * period while that is
    < horizon; a dispatched stage runs for wcet * exec_scale.  At one instant completions
    come first (in dispatch order), then releases (by task index), then dispatches.
    Returns (dispatch log, stats); a log entry is
    (time, task, job, stage, context, lane, level, deadline)."""
    s = Scheduler(n_contexts, lanes)
    for (wcet, period, D) in tasks:
        s.add_task(wcet, period, D)
    offsets = offsets or [0.0] * len(tasks)
    next_rel = list(offsets)
    active = []   # (finish, order, task, job, stage)
    order = 0
    log = []
    while True:
        times = [f for (f, *_r) in active] + [r for r in next_rel if r < horizon]
        if not times:
            break
        now = min(times)
        for ev in sorted(e for e in active if e[0] == now):
            active.remove(ev)
            s.complete(ev[2], ev[3], ev[4], now)
        for i in range(len(tasks)):
            if next_rel[i] < horizon and next_rel[i] == now:
                s.release(i, now)
                next_rel[i] = offsets[i] + s.tasks[i]["next_job"] * tasks[i][1]
        while True:
            d = s.next(now)
            if d is None:
                break
            log.append((now, d["task"], d["job"], d["stage"], d["context"], d["lane"], d["level"], d["deadline"]))
            active.append((now + d["wcet"] * exec_scale, order, d["task"], d["job"], d["stage"]))
            order += 1
    return log, dict(s.stats)
