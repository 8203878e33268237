// The SGPRS scheduler core: host-side decisions only, no GPU call and no clock of its own
// (the caller passes the time, so the same code serves a real run and a simulated one).
//
// Offline phase ("Two Level Priority Assignment", "WCET and Virtual Deadline Assignment"):
// a task's last stage is high priority, the others low; stage j gets the share
// D * C^j / sum_k C^k of the task's relative deadline.
// Online phase ("Absolute Deadline Assignment", "Context Assignment", "Stage Queuing"):
// a released stage gets the absolute deadline r + D^0 + .. + D^j (r = its job's release), is
// assigned to a context (an empty queue first, else the shortest queue among the contexts on
// which it would still meet its deadline, else the earliest finish), and waits there.  A
// context runs up to `lanes` stages at once, the first lanes / 2 lanes for high-priority
// stages, the others for medium and low ones; a low-priority stage whose predecessor missed
// its deadline is medium; inside a level the earliest deadline goes first.
#include <algorithm>
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdint>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <unordered_map>
#include <vector>

#include "internal.h"

namespace {

enum { kHigh = 0, kMedium = 1, kLow = 2 };

struct SchedTask {
    std::vector<double> wcet, vdl;
    double period = 0, deadline = 0;
    int next_job = 0;
};

struct StageRec {
    int task = 0, job = 0, stage = 0, level = kLow, context = 0, lane = -1;
    double wcet = 0, deadline = 0, start = 0;
    long long seq = 0;
};

struct JobRec {
    double release = 0;
    bool prev_missed = false;
};

struct SchedContext {
    std::vector<StageRec> waiting;
    std::vector<StageRec> running;  // one slot per lane
    std::vector<char> busy;
};

inline long long job_key(int task, int job) { return ((long long)task << 32) | (unsigned)job; }

}  // namespace

struct sgprs_sched {
    int n_contexts = 0, lanes = 0, n_high = 0;
    std::vector<SchedTask> tasks;
    std::vector<SchedContext> ctx;
    std::unordered_map<long long, JobRec> jobs;
    long long seq = 0;
    sgprs_sched_stats_t stats{};
    int max_busy = sgprs::kMaxBusyQueues;  // run loop only: lanes with a stage in flight at once (0: no limit)

    // Forgets every job in flight (after a failed run, whose stages will never be reported complete).
    void abort_jobs()
    {
        for (SchedContext& c : ctx) {
            c.waiting.clear();
            std::fill(c.busy.begin(), c.busy.end(), (char)0);
        }
        jobs.clear();
    }

    double backlog(int c, double now) const
    {
        double b = 0.0;
        for (const StageRec& s : ctx[c].waiting) b += s.wcet;
        for (int l = 0; l < lanes; ++l)
            if (ctx[c].busy[l]) b += std::max(0.0, ctx[c].running[l].wcet - (now - ctx[c].running[l].start));
        return b;
    }
    int queue_len(int c) const
    {
        int n = (int)ctx[c].waiting.size();
        for (int l = 0; l < lanes; ++l) n += ctx[c].busy[l] ? 1 : 0;
        return n;
    }
    int assign_context(double now, double wcet, double deadline) const
    {
        for (int c = 0; c < n_contexts; ++c)
            if (queue_len(c) == 0) return c;
        int best = -1;
        for (int c = 0; c < n_contexts; ++c)
            if (now + backlog(c, now) + wcet <= deadline && (best < 0 || queue_len(c) < queue_len(best))) best = c;
        if (best >= 0) return best;
        for (int c = 0; c < n_contexts; ++c)
            if (best < 0 || now + backlog(c, now) < now + backlog(best, now)) best = c;
        return best;
    }
    void release_stage(int task, int job, int stage, double now)
    {
        const SchedTask& t = tasks[task];
        const JobRec& j = jobs[job_key(task, job)];
        StageRec s;
        s.task = task; s.job = job; s.stage = stage;
        s.level = stage == (int)t.wcet.size() - 1 ? kHigh : (j.prev_missed ? kMedium : kLow);
        s.wcet = t.wcet[stage];
        double d = j.release;
        for (int k = 0; k <= stage; ++k) d += t.vdl[k];
        s.deadline = d;
        s.seq = seq++;
        s.context = assign_context(now, s.wcet, s.deadline);
        ctx[s.context].waiting.push_back(s);
    }
};

using namespace sgprs;

extern "C" {

int sgprs_sched_create(int n_contexts, int lanes_per_context, sgprs_sched_t** out)
{
    if (!out) return fail(SGPRS_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (n_contexts < 1 || n_contexts > 64) return fail(SGPRS_ERR_INVALID_ARG, "n_contexts %d outside [1,64]", n_contexts);
    if (lanes_per_context < 1 || lanes_per_context > 8)
        return fail(SGPRS_ERR_INVALID_ARG, "lanes_per_context %d outside [1,8]", lanes_per_context);
    sgprs_sched* s = new (std::nothrow) sgprs_sched;
    if (!s) return fail(SGPRS_ERR_OOM, "scheduler allocation failed");
    s->n_contexts = n_contexts;
    s->lanes = lanes_per_context;
    s->n_high = lanes_per_context / 2;
    s->ctx.resize(n_contexts);
    for (SchedContext& c : s->ctx) {
        c.running.resize(lanes_per_context);
        c.busy.assign(lanes_per_context, 0);
    }
    *out = s;
    return SGPRS_OK;
}

void sgprs_sched_destroy(sgprs_sched_t* s) { delete s; }

int sgprs_sched_add_task(sgprs_sched_t* s, int n_stages, const double* wcet, double period, double rel_deadline, int* task_id)
{
    if (!s || !wcet || !task_id) return fail(SGPRS_ERR_INVALID_ARG, "NULL argument");
    if (n_stages < 1 || n_stages > 4096) return fail(SGPRS_ERR_INVALID_ARG, "n_stages %d outside [1,4096]", n_stages);
    if (!(period > 0) || !(rel_deadline > 0)) return fail(SGPRS_ERR_INVALID_ARG, "period and deadline must be positive");
    double total = 0.0;
    for (int j = 0; j < n_stages; ++j) {
        if (!(wcet[j] > 0)) return fail(SGPRS_ERR_INVALID_ARG, "wcet[%d] must be positive", j);
        total += wcet[j];
    }
    SchedTask t;
    t.wcet.assign(wcet, wcet + n_stages);
    t.vdl.resize(n_stages);
    for (int j = 0; j < n_stages; ++j) t.vdl[j] = rel_deadline * wcet[j] / total;
    t.period = period;
    t.deadline = rel_deadline;
    s->tasks.push_back(t);
    *task_id = (int)s->tasks.size() - 1;
    return SGPRS_OK;
}

int sgprs_sched_virtual_deadlines(const sgprs_sched_t* s, int task, int capacity, double* out)
{
    if (!s || !out) return fail(SGPRS_ERR_INVALID_ARG, "NULL argument");
    if (task < 0 || task >= (int)s->tasks.size()) return fail(SGPRS_ERR_INVALID_ARG, "task %d does not exist", task);
    const SchedTask& t = s->tasks[task];
    if (capacity < (int)t.vdl.size()) return fail(SGPRS_ERR_INVALID_ARG, "capacity %d below %zu stages", capacity, t.vdl.size());
    std::copy(t.vdl.begin(), t.vdl.end(), out);
    return SGPRS_OK;
}

int sgprs_sched_release(sgprs_sched_t* s, int task, double now, int* job_id)
{
    if (!s) return fail(SGPRS_ERR_INVALID_ARG, "sched is NULL");
    if (task < 0 || task >= (int)s->tasks.size()) return fail(SGPRS_ERR_INVALID_ARG, "task %d does not exist", task);
    const int job = s->tasks[task].next_job++;
    JobRec j;
    j.release = now;
    s->jobs[job_key(task, job)] = j;
    ++s->stats.jobs_released;
    s->release_stage(task, job, 0, now);
    if (job_id) *job_id = job;
    return SGPRS_OK;
}

int sgprs_sched_next(sgprs_sched_t* s, double now, sgprs_dispatch_t* out)
{
    if (!s || !out) return fail(SGPRS_ERR_INVALID_ARG, "NULL argument");
    for (int c = 0; c < s->n_contexts; ++c) {
        SchedContext& cx = s->ctx[c];
        if (cx.waiting.empty()) continue;
        for (int lane = 0; lane < s->lanes; ++lane) {
            if (cx.busy[lane]) continue;
            int best = -1;
            for (int i = 0; i < (int)cx.waiting.size(); ++i) {
                const StageRec& w = cx.waiting[i];
                if (s->lanes > 1 && (lane < s->n_high) != (w.level == kHigh)) continue;  // lane classes
                if (best < 0) { best = i; continue; }
                const StageRec& b = cx.waiting[best];
                if (w.level != b.level ? w.level < b.level : w.deadline != b.deadline ? w.deadline < b.deadline : w.seq < b.seq)
                    best = i;
            }
            if (best < 0) continue;
            StageRec r = cx.waiting[best];
            cx.waiting.erase(cx.waiting.begin() + best);
            r.lane = lane;
            r.start = now;
            cx.running[lane] = r;
            cx.busy[lane] = 1;
            out->task = r.task; out->job = r.job; out->stage = r.stage; out->context = c; out->lane = lane;
            out->level = r.level; out->deadline = r.deadline; out->wcet = r.wcet;
            return 1;
        }
    }
    return 0;
}

int sgprs_sched_complete(sgprs_sched_t* s, int task, int job, int stage, double now, int* missed_out)
{
    if (!s) return fail(SGPRS_ERR_INVALID_ARG, "sched is NULL");
    for (int c = 0; c < s->n_contexts; ++c)
        for (int lane = 0; lane < s->lanes; ++lane) {
            SchedContext& cx = s->ctx[c];
            if (!cx.busy[lane]) continue;
            const StageRec r = cx.running[lane];
            if (r.task != task || r.job != job || r.stage != stage) continue;
            cx.busy[lane] = 0;
            const bool missed = now > r.deadline;
            ++s->stats.stages_completed;
            s->stats.stages_missed += missed ? 1 : 0;
            if (stage + 1 < (int)s->tasks[task].wcet.size()) {
                s->jobs[job_key(task, job)].prev_missed = missed;
                s->release_stage(task, job, stage + 1, now);
            } else {
                ++s->stats.jobs_completed;
                s->stats.jobs_missed += missed ? 1 : 0;
                s->jobs.erase(job_key(task, job));
            }
            if (missed_out) *missed_out = missed ? 1 : 0;
            return SGPRS_OK;
        }
    return fail(SGPRS_ERR_INVALID_ARG, "stage %d of job %d of task %d is not running", stage, job, task);
}

int sgprs_sched_set_max_busy(sgprs_sched_t* s, int max_busy)
{
    if (!s) return fail(SGPRS_ERR_INVALID_ARG, "sched is NULL");
    if (max_busy < 0) return fail(SGPRS_ERR_INVALID_ARG, "max_busy %d < 0", max_busy);
    s->max_busy = max_busy;
    return SGPRS_OK;
}

int sgprs_sched_get_stats(const sgprs_sched_t* s, sgprs_sched_stats_t* out)
{
    if (!s || !out) return fail(SGPRS_ERR_INVALID_ARG, "NULL argument");
    *out = s->stats;
    return SGPRS_OK;
}

// The periodic-release experiment of "Simulation Results" on the real pool: one host thread
// releases the jobs, asks the scheduler what may start, enqueues those stages on the lane's
// partition and polls one event per lane for completions.
int sgprs_sched_run_periodic(sgprs_sched_t* s, sgprs_pool_t* pool, sgprs_task_t* const* tasks, int n_tasks,
                             const void* const* inputs, float* const* logits, int batch, const double* offsets,
                             double duration_s, sgprs_run_report_t* report)
{
    if (!s || !pool || !tasks || !inputs || !logits || !report) return fail(SGPRS_ERR_INVALID_ARG, "NULL argument");
    if (n_tasks != (int)s->tasks.size()) return fail(SGPRS_ERR_INVALID_ARG, "%d tasks given, the scheduler knows %zu", n_tasks, s->tasks.size());
    if (!(duration_s > 0) || duration_s > 600) return fail(SGPRS_ERR_INVALID_ARG, "duration_s outside (0,600]");
    if (!s->jobs.empty()) return fail(SGPRS_ERR_INVALID_ARG, "the scheduler still has jobs in flight");
    int n_p = 0, cpp = 0, total = 0, nx = 0, rc;
    if ((rc = sgprs_pool_info(pool, &n_p, &cpp, &total, &nx))) return rc;
    if (n_p < s->n_contexts * s->lanes)
        return fail(SGPRS_ERR_INVALID_ARG, "the pool has %d partitions, %d contexts x %d lanes need %d", n_p, s->n_contexts, s->lanes,
                    s->n_contexts * s->lanes);
    for (int i = 0; i < n_tasks; ++i) {
        if (!tasks[i] || !inputs[i] || !logits[i]) return fail(SGPRS_ERR_INVALID_ARG, "task %d: NULL handle or buffer", i);
        if (sgprs_task_num_stages(tasks[i]) != (int)s->tasks[i].wcet.size())
            return fail(SGPRS_ERR_INVALID_ARG, "task %d has %d stages, the scheduler knows %zu", i, sgprs_task_num_stages(tasks[i]),
                        s->tasks[i].wcet.size());
    }
    // One slot per lane.  The scheduling thread owns `busy` and the ids; the launch itself (a handful
    // of kernel launches and the event record, 20-30 us of host time) is done by the lane's own
    // launcher thread, so that one slow enqueue does not hold up the decisions for the other lanes.
    struct Slot {
        bool busy = false;
        int task = 0, job = 0, stage = 0;
        hipEvent_t ev = nullptr;
        hipStream_t stream = nullptr;
        std::atomic<int> state{0};  // 0 idle, 1 launch requested, 2 launched (event recorded), 3 launch failed, 4 quit
        std::mutex mu;              // the launcher thread sleeps on cv until state becomes 1 or 4
        std::condition_variable cv;
        sgprs_task_t* rq_task = nullptr;
        const void* rq_in = nullptr;
        void* rq_out = nullptr;
        int rq_partition = 0, rc = 0;
        std::string error;
        std::thread thread;
    };
    const size_t n_slots = (size_t)s->n_contexts * s->lanes;
    std::unique_ptr<Slot[]> slots(new (std::nothrow) Slot[n_slots]);
    if (!slots) return fail(SGPRS_ERR_OOM, "slot allocation failed");
    const bool threaded = n_slots <= 16;  // beyond that the scheduling thread launches by itself
    int device = 0;
    (void)hipGetDevice(&device);
    auto launch = [&](Slot& sl) {
        sl.rc = sgprs_stage_run(sl.rq_task, sl.stage, batch, sl.rq_in, sl.rq_out, pool, sl.rq_partition);
        if (!sl.rc && hipEventRecord(sl.ev, sl.stream) != hipSuccess) sl.rc = fail(SGPRS_ERR_HIP, "hipEventRecord failed");
        if (sl.rc) sl.error = sgprs_last_error();
        sl.state.store(sl.rc ? 3 : 2, std::memory_order_release);
    };
    auto launcher = [&](Slot* sl) {   // blocks between requests: idle lanes cost no host core
        (void)hipSetDevice(device);
        for (;;) {
            int st;
            {
                std::unique_lock<std::mutex> lk(sl->mu);
                sl->cv.wait(lk, [&] { const int v = sl->state.load(std::memory_order_acquire); return v == 1 || v == 4; });
                st = sl->state.load(std::memory_order_acquire);
            }
            if (st == 4) return;
            launch(*sl);
        }
    };
    auto post = [&](Slot& sl, int st) {   // hands a request (1) or the quit order (4) to the lane's launcher
        {
            std::lock_guard<std::mutex> lk(sl.mu);
            sl.state.store(st, std::memory_order_release);
        }
        sl.cv.notify_one();
    };
    auto cleanup = [&]() {
        for (size_t p = 0; p < n_slots; ++p) {
            Slot& sl = slots[p];
            if (sl.thread.joinable()) {
                while (sl.state.load(std::memory_order_acquire) == 1) std::this_thread::yield();  // a launch in progress finishes first
                post(sl, 4);
                sl.thread.join();
            }
            if (sl.busy && sl.state.load() != 3 && sl.ev) (void)hipEventSynchronize(sl.ev);  // nothing of ours stays queued unseen
            if (sl.ev) (void)hipEventDestroy(sl.ev);
        }
    };
    for (size_t p = 0; p < n_slots; ++p) {
        slots[p].stream = (hipStream_t)sgprs_pool_stream(pool, (int)p);
        if (hipEventCreateWithFlags(&slots[p].ev, hipEventDisableTiming) != hipSuccess) {
            cleanup();
            return fail(SGPRS_ERR_HIP, "hipEventCreateWithFlags failed");
        }
    }
    if (threaded)
        for (size_t p = 0; p < n_slots; ++p) slots[p].thread = std::thread(launcher, &slots[p]);
    std::vector<long long> released(n_tasks, 0);
    std::vector<char> active(n_tasks, 0);
    std::vector<double> job_release(n_tasks, 0.0);
    const sgprs_sched_stats_t before = s->stats;
    long long releases = 0, dropped = 0, in_flight = 0;
    int busy_lanes = 0;
    double resp_sum = 0.0, resp_max = 0.0, last_done = 0.0;
    const auto t0 = std::chrono::steady_clock::now();
    auto clock_s = [&]() { return std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count(); };
    int status = SGPRS_OK;
    for (;;) {
        const double now = clock_s();
        // completions
        for (size_t p = 0; p < n_slots; ++p) {
            Slot& sl = slots[p];
            if (!sl.busy) continue;
            const int st = sl.state.load(std::memory_order_acquire);
            if (st == 1) continue;  // its launcher is still enqueueing
            if (st == 3) { status = fail(sl.rc, "%s", sl.error.c_str()); break; }
            const hipError_t q = hipEventQuery(sl.ev);
            if (q == hipErrorNotReady) continue;
            if (q != hipSuccess) { status = fail(SGPRS_ERR_HIP, "hipEventQuery: %s", hipGetErrorString(q)); break; }
            sl.busy = false;
            --busy_lanes;
            sl.state.store(0, std::memory_order_relaxed);
            if ((status = sgprs_sched_complete(s, sl.task, sl.job, sl.stage, now, nullptr))) break;
            if (sl.stage + 1 == (int)s->tasks[sl.task].wcet.size()) {
                active[sl.task] = 0;
                --in_flight;
                const double r = now - job_release[sl.task];
                resp_sum += r;
                resp_max = std::max(resp_max, r);
                last_done = now;
            }
        }
        if (status) break;
        // releases: job k of task i at offsets[i] + k * period; a job whose predecessor is still in
        // flight is dropped (the task's buffers hold one job at a time) and counted as a miss
        bool more_releases = false;
        for (int i = 0; i < n_tasks; ++i) {
            for (;;) {
                const double r = (offsets ? offsets[i] : 0.0) + (double)released[i] * s->tasks[i].period;
                if (r >= duration_s) break;
                more_releases = true;
                if (r > now) break;
                ++released[i];
                ++releases;
                if (active[i]) { ++dropped; continue; }
                if ((status = sgprs_sched_release(s, i, r, nullptr))) break;
                active[i] = 1;
                job_release[i] = r;
                ++in_flight;
            }
            if (status) break;
        }
        if (status) break;
        // dispatches
        // (at most max_busy lanes have a stage in flight: more CU-masked streams busy at once than the
        // device has hardware queues for one process collapse the throughput of all of them, so further
        // stages wait in the scheduler's queues even if their lane is free)
        sgprs_dispatch_t d;
        int got = 0;
        while ((s->max_busy <= 0 || busy_lanes < s->max_busy) && (got = sgprs_sched_next(s, now, &d)) == 1) {
            Slot& sl = slots[(size_t)d.context * s->lanes + d.lane];
            const int last = (int)s->tasks[d.task].wcet.size() - 1;
            const void* in = d.stage == 0 ? inputs[d.task] : sgprs_task_stage_output(tasks[d.task], d.stage - 1);
            void* out = d.stage == last ? (void*)logits[d.task] : (void*)sgprs_task_stage_output(tasks[d.task], d.stage);
            sl.busy = true; sl.task = d.task; sl.job = d.job; sl.stage = d.stage;
            sl.rq_task = tasks[d.task]; sl.rq_in = in; sl.rq_out = out; sl.rq_partition = d.context * s->lanes + d.lane;
            ++busy_lanes;
            if (threaded) post(sl, 1);
            else {
                launch(sl);
                if (sl.rc) { status = fail(sl.rc, "%s", sl.error.c_str()); break; }
            }
        }
        if (got < 0) status = got;
        if (status) break;
        if (!more_releases && in_flight == 0) break;
        if (now > duration_s + 30.0) { status = fail(SGPRS_ERR_HIP, "jobs still in flight 30 s after the last release"); break; }
    }
    cleanup();
    if (status) {
        s->abort_jobs();   // nothing of this run stays in the scheduler: the next run starts clean
        return status;
    }
    report->elapsed_s = std::max(last_done, duration_s);
    report->releases = releases;
    report->dropped = dropped;
    report->sched.jobs_released = s->stats.jobs_released - before.jobs_released;
    report->sched.jobs_completed = s->stats.jobs_completed - before.jobs_completed;
    report->sched.jobs_missed = s->stats.jobs_missed - before.jobs_missed;
    report->sched.stages_completed = s->stats.stages_completed - before.stages_completed;
    report->sched.stages_missed = s->stats.stages_missed - before.stages_missed;
    report->fps = (double)report->sched.jobs_completed / report->elapsed_s;
    report->dmr = releases ? (double)(report->sched.jobs_missed + dropped) / (double)releases : 0.0;
    report->mean_response_s = report->sched.jobs_completed ? resp_sum / (double)report->sched.jobs_completed : 0.0;
    report->max_response_s = resp_max;
    return SGPRS_OK;
}

// Static (purely spatial) execution: every task keeps the partition it is given; the calling thread
// hands out whole inferences and polls one event per task, with the same gate on busy partitions.
int sgprs_pool_run_static(sgprs_pool_t* pool, sgprs_task_t* const* tasks, int n_tasks, const void* const* inputs,
                          float* const* logits, int batch, const int* partition_of_task, int rounds, int max_busy,
                          double* elapsed_s)
{
    if (!pool || !tasks || !inputs || !logits || !partition_of_task) return fail(SGPRS_ERR_INVALID_ARG, "NULL argument");
    if (n_tasks <= 0 || n_tasks > 4096 || rounds <= 0 || max_busy < 0) return fail(SGPRS_ERR_INVALID_ARG, "n_tasks, rounds or max_busy out of range");
    int n_p = 0, rc;
    if ((rc = sgprs_pool_info(pool, &n_p, nullptr, nullptr, nullptr))) return rc;
    for (int i = 0; i < n_tasks; ++i) {
        if (!tasks[i] || !inputs[i] || !logits[i]) return fail(SGPRS_ERR_INVALID_ARG, "task %d: NULL handle or buffer", i);
        if (partition_of_task[i] < 0 || partition_of_task[i] >= n_p) return fail(SGPRS_ERR_INVALID_ARG, "task %d: partition %d outside the pool", i, partition_of_task[i]);
    }
    std::vector<hipEvent_t> ev(n_tasks, nullptr);
    auto cleanup = [&]() {
        for (hipEvent_t e : ev)
            if (e) { (void)hipEventSynchronize(e); (void)hipEventDestroy(e); }
    };
    for (int i = 0; i < n_tasks; ++i)
        if (hipEventCreateWithFlags(&ev[i], hipEventDisableTiming) != hipSuccess) {
            ev[i] = nullptr;
            cleanup();
            return fail(SGPRS_ERR_HIP, "hipEventCreateWithFlags failed");
        }
    std::vector<int> done(n_tasks, 0);
    std::vector<char> running(n_tasks, 0), part_busy(n_p, 0);
    int busy = 0, finished = 0, status = SGPRS_OK, next = 0;
    const auto t0 = std::chrono::steady_clock::now();
    while (finished < n_tasks && !status) {
        for (int i = 0; i < n_tasks && !status; ++i) {
            if (!running[i]) continue;
            const hipError_t q = hipEventQuery(ev[i]);
            if (q == hipErrorNotReady) continue;
            if (q != hipSuccess) { status = fail(SGPRS_ERR_HIP, "hipEventQuery: %s", hipGetErrorString(q)); break; }
            running[i] = 0;
            part_busy[partition_of_task[i]] = 0;
            --busy;
            if (++done[i] == rounds) ++finished;
        }
        // hand out work round-robin, starting behind the task served last
        for (int k = 0; k < n_tasks && !status && (max_busy == 0 || busy < max_busy); ++k) {
            const int i = (next + k) % n_tasks, p = partition_of_task[i];
            if (running[i] || done[i] == rounds || part_busy[p]) continue;
            if ((status = sgprs_task_run(tasks[i], batch, inputs[i], logits[i], pool, p, nullptr))) break;
            if (hipEventRecord(ev[i], (hipStream_t)sgprs_pool_stream(pool, p)) != hipSuccess) { status = fail(SGPRS_ERR_HIP, "hipEventRecord failed"); break; }
            running[i] = 1;
            part_busy[p] = 1;
            ++busy;
            next = (i + 1) % n_tasks;
        }
    }
    cleanup();   // (waits for whatever is still queued)
    if (status) return status;
    if (elapsed_s) *elapsed_s = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    return SGPRS_OK;
}

}  // extern "C"
