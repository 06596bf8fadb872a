// Bubble-harvesting runtime: side-task state machine, worker thread, step planning loop, memory accounting,
// event log.  Follows FreeRide (arXiv 2409.06941): Section 4.1 (states and transitions), Section 4.4
// (Algorithm 1: admission by memory; Algorithm 2: bubble -> Init / Start / Pause), Section 4.5 (program-directed
// time limit and the framework-enforced limit with its grace period, memory limit).  The paper's manager / worker /
// task processes are one worker thread here; a task that the paper would kill is stopped and its memory released.

#include <time.h>

#include <atomic>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <thread>

#include "common.h"
#include "freeride_device.h"

namespace {

// ---- device gate (freeride_device.h): opened at the start of every bubble the task runs in
__global__ void k_gate_open(fr_gate* g, unsigned long long deadline_ticks)
{
    g->deadline_ticks = deadline_ticks;
    g->opened_ticks = wall_clock64();
    g->end_ticks[0] = g->end_ticks[1] = 0ull;
    g->state = FR_GATE_OPEN;
    g->tiles_done = 0u;
}

__global__ void k_gate_clock(fr_gate* g) { g->deadline_ticks = wall_clock64(); }

inline void cpu_relax()
{
    __builtin_ia32_pause();
}

// GPU time is measured between two events around a group of consecutive steps (time_steps steps per group; an
// event between two kernels costs about 3 us of GPU idle time, so timing every step is for profiling passes).
// Inside a bubble the groups form a chain: the end event of one group is the begin event of the next, so the
// measured times add up to the chain's span.
struct PendingTiming {
    uint64_t log_seq;        // sequence number of the group's last CHUNK record, which receives the measured time
    hipEvent_t begin;
    hipEvent_t end;
    uint32_t class_mask;     // for cost adaptation: the cost classes in the group and the task's own (unscaled)
    uint64_t task_modelled_ns;   // modelled cost of its steps
    uint64_t bubble;         // index of the bubble the group ran in
    void* owner;             // the task whose steps these are (it may no longer be the current one when they resolve)
};

// Cost adaptation gathers the timing groups of a bubble and updates the scales once from the bubble's totals: single
// groups scatter by several percent (the first after a burst of the main workload runs slowest), and a scale that
// follows every group ends up charging every step for the slowest one.
struct BubbleTotals {
    uint64_t bubble = ~0ull;
    uint64_t modelled_ns[8] = {}, measured_ns[8] = {};       // per cost class: of the groups that hold steps of it
    bool surged = false;         // a group far over its cost has raised the scales for the rest of this bubble ...
    uint32_t before_surge[8];    // ... from these values, which the bubble's totals then update
};

constexpr uint32_t kScaleOne = 1000000, kScaleMin = 250000, kScaleMax = 16000000;

struct Task {
    fr_task_ops ops{};
    void* user = nullptr;
    fr_task_profile prof{};
    fr_task_id id = 0;
    int state = FR_SUBMITTED;
    int last_error = FR_OK;
    fr_alloc alloc;
    fr_progress prog{};
};

}  // namespace

struct fr_ctx {
    fr_config cfg{};
    bool host_only = false;
    hipStream_t side = nullptr;
    int hip_error = 0;

    std::mutex mu;                 // guards task, progress, log
    std::mutex work_mu;            // held by the worker while it runs task callbacks for a bubble
    std::thread worker;
    std::atomic<bool> quit{false};
    std::atomic<bool> abort_steps{false};   // fr_task_stop / fr_destroy ask the step loop to leave

    // bubble hand-off (stage thread -> worker)
    std::atomic<uint64_t> bubble_seq{0};    // bumped by fr_bubble_begin after the fields below are written
    std::atomic<uint64_t> ack_seq{0};       // worker: "I will enqueue nothing more for bubble ack_seq"
    std::atomic<bool> end_requested{false};
    std::atomic<bool> in_init{false};       // the worker is inside the task's init()
    std::atomic<uint64_t> in_callback{0};   // nonzero: the worker is inside plan_step / run_step since that time
    // Framework-enforced limit (Section 4.5): armed when a bubble ends with side work still going on (on the GPU,
    // or a callback that has not returned); if the work is still going on `grace_ns` later the task is killed.
    std::atomic<bool> kill_current{false};  // the worker stops the current task the next time it is between callbacks
    bool enforce_armed = false;             // stage thread only
    bool enforce_gpu = false;               //   what is late: GPU work behind tail_event, or a host callback
    uint64_t enforce_callback = 0;          //   the late callback's start time (identifies it)
    uint64_t enforce_deadline = 0;
    bool bubble_open = false;               // stage thread only
    // (written by the stage thread before bubble_seq is bumped; the worker reads them, checks that bubble_seq has not
    // moved meanwhile and reads again if it has: a bubble may open while the worker is still closing the one before)
    std::atomic<uint64_t> cur_begin{0}, cur_len{0};
    std::atomic<uint32_t> cur_index{0};     // 0-based bubble index
    uint64_t bubbles_total = 0;

    Task* task = nullptr;                   // the worker's current task (Algorithm 2)
    std::deque<Task*> queue;                // accepted tasks waiting their turn (Algorithm 1 appends, Algorithm 2 pops)
    std::vector<Task*> tasks;               // every task registered with this context, owned
    fr_task_id next_id = 1;

    // event log ring
    std::vector<fr_event> log;
    uint64_t log_first_seq = 0;             // sequence number of log[log_head]
    size_t log_head = 0, log_count = 0;

    // step timing
    std::vector<hipEvent_t> free_events;
    std::deque<PendingTiming> pending;
    hipEvent_t chain_tail = nullptr;        // end event of the newest step of the bubble being served
    uint32_t cost_scale[8] = {kScaleOne, kScaleOne, kScaleOne, kScaleOne, kScaleOne, kScaleOne, kScaleOne, kScaleOne};
    BubbleTotals totals;     // of the bubble whose timing groups are being resolved

    // device gate
    fr_gate* gate = nullptr;                // device memory, NULL when the gate is off
    double ticks_per_ns = 0.0;              // GPU wall clock
    int64_t gpu_minus_host_ns = 0;          // wall_clock64() / ticks_per_ns - CLOCK_MONOTONIC
    uint64_t clock_window_ns = 0;           // width of the window that reading came from
    uint64_t clock_read_ns = 0;             // host time of that reading
    std::vector<fr_step> gate_steps;        // steps enqueued since the gate was last opened, by slot (worker only)
    std::vector<uint32_t> gate_bubble;      //   and the bubble each belongs to
    std::vector<uint64_t> gate_seq;         //   and the sequence number of its CHUNK record
    std::atomic<bool> gate_pending{false};  // their verdicts have not been read back yet

    // Overrun detection: the worker records this event behind the last work it enqueued for a bubble;
    // fr_bubble_end asks whether it has completed.  (A stream query is not used: it may report "not ready"
    // for a stream whose last command carries no completion signal, although all work has finished.)
    hipEvent_t tail_event = nullptr;
    bool tail_armed = false;                // written by the worker before ack_seq, read after it
};

namespace {

uint64_t now_ns()
{
    timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return (uint64_t)ts.tv_sec * 1000000000ull + (uint64_t)ts.tv_nsec;
}

// ---- log (ctx->mu held) ----
uint64_t log_push(fr_ctx* c, const fr_event& ev)
{
    const size_t cap = c->log.size();
    uint64_t seq = c->log_first_seq + c->log_count;
    if (c->log_count == cap) {            // drop the oldest
        c->log_head = (c->log_head + 1) % cap;
        c->log_first_seq++;
        c->log_count--;
    }
    c->log[(c->log_head + c->log_count) % cap] = ev;
    c->log_count++;
    return seq;
}

fr_event* log_at(fr_ctx* c, uint64_t seq)
{
    if (seq < c->log_first_seq || seq >= c->log_first_seq + c->log_count) return nullptr;
    return &c->log[(c->log_head + (seq - c->log_first_seq)) % c->log.size()];
}

hipEvent_t event_get(fr_ctx* c)
{
    if (!c->free_events.empty()) {
        hipEvent_t e = c->free_events.back();
        c->free_events.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// The scales take in what the finished bubble showed (ctx->mu held).
void apply_totals(fr_ctx* c)
{
    BubbleTotals& b = c->totals;
    if (b.surged) {
        for (int k = 0; k < 8; ++k) c->cost_scale[k] = b.before_surge[k];
        b.surged = false;
    }
    for (int k = 0; k < 8; ++k) {
        if (b.modelled_ns[k]) c->cost_scale[k] = fr_cost_scale_next(c->cost_scale[k], b.modelled_ns[k], b.measured_ns[k]);
        b.modelled_ns[k] = b.measured_ns[k] = 0;
    }
}

// Resolve finished step timings (ctx->mu held).  wait = true blocks until every pending step has finished.
void resolve_timings(fr_ctx* c, bool wait)
{
    while (!c->pending.empty()) {
        PendingTiming& p = c->pending.front();
        hipError_t q = wait ? hipEventSynchronize(p.end) : hipEventQuery(p.end);
        if (q == hipErrorNotReady) break;
        float ms = 0.f;
        if (q == hipSuccess && hipEventElapsedTime(&ms, p.begin, p.end) == hipSuccess) {
            const uint64_t ns = (uint64_t)((double)ms * 1.0e6 + 0.5);
            if (fr_event* ev = log_at(c, p.log_seq)) ev->measured_ns = ns;
            for (Task* t : c->tasks)
                if (t == p.owner) t->prog.ns_measured += ns;
            if (c->cfg.adapt_costs) {
                if (p.bubble != c->totals.bubble) { apply_totals(c); c->totals.bubble = p.bubble; }
                // a group that took over 1.25 times its scaled cost is no scatter: the steps still to be planned for
                // this bubble are charged more at once.  What stays after the bubble is what its totals say, this
                // group included: a model that is wrong shows there too, a hiccup does not weigh much
                bool far_off = false;
                for (int k = 0; k < 8; ++k)
                    if ((p.class_mask >> k) & 1u)
                        far_off |= (unsigned __int128)ns * kScaleOne * 4 > (unsigned __int128)p.task_modelled_ns * c->cost_scale[k] * 5;
                if (far_off) {
                    if (!c->totals.surged) {
                        for (int k = 0; k < 8; ++k) c->totals.before_surge[k] = c->cost_scale[k];
                        c->totals.surged = true;
                    }
                    for (int k = 0; k < 8; ++k)
                        if ((p.class_mask >> k) & 1u) c->cost_scale[k] = fr_cost_scale_next(c->cost_scale[k], p.task_modelled_ns, ns);
                }
                for (int k = 0; k < 8; ++k)
                    if ((p.class_mask >> k) & 1u) { c->totals.modelled_ns[k] += p.task_modelled_ns; c->totals.measured_ns[k] += ns; }
            }
        }
        // Steps resolve in order, so nothing older still needs this begin event.  The end event lives on if a
        // later step uses (or may still come to use) it as its begin; that step releases it.
        c->free_events.push_back(p.begin);
        const bool next_begins_here = c->pending.size() > 1 && c->pending[1].begin == p.end;
        if (p.end != c->chain_tail && !next_begins_here) c->free_events.push_back(p.end);
        c->pending.pop_front();
    }
}

void stop_task_locked(fr_ctx* c, Task* t, int error)
{
    // ctx->mu held, work_mu held by the caller or caller is the worker itself
    if (t->state == FR_STOPPED) return;
    if (!c->host_only && c->side) (void)hipStreamSynchronize(c->side);
    resolve_timings(c, true);
    if (t->ops.stop) t->ops.stop(t->user);
    if (t == c->task) { c->gate_steps.clear(); c->gate_bubble.clear(); c->gate_seq.clear(); c->gate_pending = false; }
    t->prog.mem_used_bytes = t->alloc.used;
    fr_alloc_release(&t->alloc);
    t->state = FR_STOPPED;
    if (error != FR_OK) t->last_error = error;
}

// Algorithm 2: when the worker has no live current task, the next one in its queue becomes current and is
// created.  ctx->mu and work_mu held.
void promote_locked(fr_ctx* c)
{
    while ((!c->task || c->task->state == FR_STOPPED) && !c->queue.empty()) {
        Task* t = c->queue.front();
        c->queue.pop_front();
        const int rc = t->ops.create ? t->ops.create(t->user) : FR_OK;      // CreateSideTask()
        if (rc != FR_OK) { t->state = FR_STOPPED; t->last_error = rc; continue; }
        t->state = FR_CREATED;
        c->task = t;
        for (int k = 0; k < 8; ++k) c->cost_scale[k] = kScaleOne;     // what the task before taught says nothing about this one
        c->totals = BubbleTotals{};
    }
}

Task* find_task(fr_ctx* c, fr_task_id id)
{
    for (Task* t : c->tasks)
        if (t->id == id) return t;
    return nullptr;
}

// The framework-enforced limit has expired for the current task: stop it, as the paper's worker kills the
// task's process, and let the next queued task take its place.  Worker thread, work_mu held.
bool killed_if_asked(fr_ctx* c, Task* t)
{
    if (!c->kill_current.load(std::memory_order_acquire)) return false;
    std::lock_guard<std::mutex> lk(c->mu);
    c->kill_current.store(false, std::memory_order_release);
    if (t->state != FR_STOPPED) {
        t->prog.killed = 1;
        stop_task_locked(c, t, FR_ERR_OVERRUN);
        promote_locked(c);
    }
    return true;
}

// Reads back where the device gate cut the bubble's steps off and takes back what was not done: the task's cursor
// is rewound to the first tile not done, the counters forget it and one FR_EV_REFUSED record is written for each
// step concerned (a step that stopped between tiles keeps its CHUNK record, shortened to the tiles it did).  Waits
// for the side stream (its work belongs to a bubble that is over).  Worker thread, work_mu held, ctx->mu not held.
void gate_settle(fr_ctx* c, Task* t)
{
    if (!c->gate_pending.exchange(false)) return;
    fr_gate g{};
    g.state = FR_GATE_OPEN;
    if (hipStreamSynchronize(c->side) != hipSuccess || hipMemcpy(&g, c->gate, sizeof(g), hipMemcpyDeviceToHost) != hipSuccess)
        g.state = FR_GATE_OPEN;
    const size_t first = g.state == FR_GATE_OPEN ? c->gate_steps.size() : (size_t)(g.state >> 1);
    if (first < c->gate_steps.size() && t && t->state != FR_STOPPED && t->ops.rewind) {
        const fr_step& cut = c->gate_steps[first];
        uint32_t done = (g.state & 1u) ? g.tiles_done : 0u;
        if (done > cut.tile1 - cut.tile0) done = cut.tile1 - cut.tile0;       // (cannot happen)
        uint64_t work_done = 0;
        const int rc = t->ops.rewind(t->user, &cut, done, &work_done);
        std::lock_guard<std::mutex> lk(c->mu);
        for (size_t i = first; i < c->gate_steps.size(); ++i) {
            const fr_step& st = c->gate_steps[i];
            const bool partly = i == first && done > 0;
            fr_event ev{};
            ev.kind = FR_EV_REFUSED; ev.bubble = c->gate_bubble[i]; ev.run = st.run; ev.segment = st.segment;
            ev.tile0 = st.tile0 + (partly ? done : 0u); ev.tile1 = st.tile1;
            ev.work_units = st.work_units - (partly ? work_done : 0); ev.t_host_ns = now_ns();
            log_push(c, ev);
            t->prog.steps_refused++;
            t->prog.work_units_done -= ev.work_units;
            if (partly) {
                if (fr_event* chunk = log_at(c, c->gate_seq[i])) { chunk->tile1 = ev.tile0; chunk->work_units = work_done; }
            } else {
                t->prog.steps--;
            }
            if (st.completes_run) t->prog.runs_completed--;
        }
        if (rc != FR_OK) { stop_task_locked(c, t, rc); promote_locked(c); }
    }
    c->gate_steps.clear();
    c->gate_bubble.clear();
    c->gate_seq.clear();
}

void gate_refresh_clock(fr_ctx* c);

// One bubble, on the worker thread, work_mu held.
void serve_bubble(fr_ctx* c, uint64_t seq, uint64_t t_begin, uint64_t len, uint32_t index)
{
    Task* t;
    {
        std::lock_guard<std::mutex> lk(c->mu);
        t = c->task;
        if (!t) return;
        t->prog.bubbles_seen++;
        t->prog.ns_bubble_declared += len;
    }
    // (a newer bubble_seq: this bubble was closed without the worker's acknowledgement and the next one is open)
    auto stop_now = [&]() {
        return c->end_requested.load(std::memory_order_acquire) || c->abort_steps.load() || c->quit.load() ||
               c->bubble_seq.load(std::memory_order_acquire) != seq;
    };
    if (killed_if_asked(c, t)) return;

    if (t->state == FR_CREATED) {
        // Algorithm 2: a CREATED current task is initialised by the new bubble.
        c->in_init.store(true, std::memory_order_release);
        int rc = t->ops.init ? t->ops.init(t->user, &t->alloc, (void*)c->side) : FR_OK;
        c->in_init.store(false, std::memory_order_release);
        std::lock_guard<std::mutex> lk(c->mu);
        fr_event ev{};
        ev.kind = FR_EV_INIT; ev.bubble = index; ev.t_host_ns = now_ns();
        log_push(c, ev);
        t->prog.mem_used_bytes = t->alloc.used;
        if (t->alloc.oom) stop_task_locked(c, t, FR_ERR_OOM);
        else if (rc != FR_OK) {
            if (rc == FR_ERR_HIP) c->hip_error = t->alloc.hip_error ? t->alloc.hip_error : c->hip_error;
            stop_task_locked(c, t, rc);
        } else if (c->kill_current.exchange(false)) {
            t->prog.killed = 1;                          // the initialisation outlived its bubble and the grace period
            stop_task_locked(c, t, FR_ERR_OVERRUN);
        } else t->state = FR_PAUSED;
        if (t->state == FR_STOPPED) promote_locked(c);
        if (!c->host_only && c->tail_event && t->state == FR_PAUSED)
            c->tail_armed = hipEventRecord(c->tail_event, c->side) == hipSuccess;
        return;
    }
    if (t->state != FR_PAUSED) return;

    {   // StartSideTask(): the task learns the bubble's end time
        std::lock_guard<std::mutex> lk(c->mu);
        t->state = FR_RUNNING;
    }
    const uint64_t guard = c->cfg.guard_ns, launch = c->cfg.launch_cost_ns;
    const uint64_t max_chunk = c->cfg.max_chunk_ns ? c->cfg.max_chunk_ns : ~0ull;
    const uint32_t max_inflight = c->cfg.max_inflight ? c->cfg.max_inflight : 8;
    const bool timed = c->cfg.time_steps && !c->host_only;
    const bool adapt = timed && c->cfg.adapt_costs;
    const bool gated = c->gate && t->ops.rewind;
    if (adapt) {                                             // what the bubble before showed goes into this one's plan
        std::lock_guard<std::mutex> lk(c->mu);
        resolve_timings(c, false);
        if (c->totals.bubble != index) apply_totals(c);
    }
    if (gated) {
        gate_settle(c, t);                                   // the previous bubble's verdicts, if still unread
        if (t->state != FR_RUNNING) return;                  // a failing rewind stopped the task
        gate_refresh_clock(c);
        const uint64_t gate_guard = c->cfg.gate_guard_ns ? c->cfg.gate_guard_ns : guard;
        const int64_t end_gpu_ns = (int64_t)(t_begin + len) - (int64_t)gate_guard + c->gpu_minus_host_ns;
        const unsigned long long deadline = end_gpu_ns > 0 ? (unsigned long long)((double)end_gpu_ns * c->ticks_per_ns) : 0ull;
        hipLaunchKernelGGL(k_gate_open, dim3(1), dim3(1), 0, c->side, c->gate, deadline);
    }
    int64_t remaining = (int64_t)len - (int64_t)guard;
    const int64_t total = remaining;
    bool used = false, finished = false;
    int fail = FR_OK;
    // the group of steps being timed together
    const uint32_t group_size = c->cfg.time_steps ? c->cfg.time_steps : 1;
    uint32_t group_n = 0, group_mask = 0;
    uint64_t group_modelled = 0, group_last_seq = 0;
    hipEvent_t group_begin = nullptr;
    auto close_group = [&]() {
        // an end event behind the group's last step; the interval goes to that step's record
        hipEvent_t ev_end;
        { std::lock_guard<std::mutex> lk(c->mu); ev_end = event_get(c); }
        if (ev_end && group_begin && hipEventRecord(ev_end, c->side) == hipSuccess) {
            std::lock_guard<std::mutex> lk(c->mu);
            c->pending.push_back(PendingTiming{group_last_seq, group_begin, ev_end, group_mask, group_modelled, index, t});
            c->chain_tail = ev_end;
        }
        group_n = 0; group_mask = 0; group_modelled = 0; group_begin = nullptr;
    };

    while (!stop_now()) {
        const uint64_t budget = remaining > 0 ? ((uint64_t)remaining < max_chunk ? (uint64_t)remaining : max_chunk) : 0;
        fr_step st{};
        c->in_callback.store(now_ns(), std::memory_order_release);
        int rc = t->ops.plan_step(t->user, budget, launch, &st);
        c->in_callback.store(0, std::memory_order_release);
        if (rc != FR_OK) { fail = rc; break; }
        if (c->kill_current.load(std::memory_order_acquire)) break;
        if (st.finished) { finished = true; break; }
        uint64_t scaled = st.modelled_ns;
        if (adapt && st.modelled_ns) {
            // plan against the scaled cost: if the step the task offers no longer fits once scaled, ask again
            // with a budget shrunk by the same factor (plan_step is pure, so asking twice is harmless)
            uint32_t scale;
            { std::lock_guard<std::mutex> lk(c->mu); resolve_timings(c, false); scale = c->cost_scale[st.cost_class & 7]; }
            auto scale_up = [&](uint64_t ns) { return (uint64_t)(((unsigned __int128)ns * scale + kScaleOne - 1) / kScaleOne); };
            scaled = scale_up(st.modelled_ns);
            if (scaled + launch > budget) {
                const uint64_t room = budget > launch ? (uint64_t)(((unsigned __int128)(budget - launch) * kScaleOne) / scale) : 0;
                c->in_callback.store(now_ns(), std::memory_order_release);
                rc = t->ops.plan_step(t->user, room + launch, launch, &st);
                c->in_callback.store(0, std::memory_order_release);
                if (rc != FR_OK) { fail = rc; break; }
                scaled = scale_up(st.modelled_ns);
                if (scaled + launch > budget) st.modelled_ns = 0;       // rounding: treat as "does not fit"
            }
        }
        if (st.modelled_ns == 0) {
            // the remaining time is not enough for the next step: leave the rest of the bubble idle
            std::lock_guard<std::mutex> lk(c->mu);
            fr_event ev{};
            ev.kind = FR_EV_IDLE; ev.bubble = index; ev.run = st.run; ev.segment = st.segment;
            ev.tile0 = st.tile0; ev.tile1 = st.tile0;
            ev.modelled_ns = remaining > 0 ? (uint64_t)remaining : 0; ev.t_host_ns = now_ns();
            log_push(c, ev);
            t->prog.ns_idle_insufficient += ev.modelled_ns;
            break;
        }
        const uint64_t cost = scaled + launch;
        // real-clock check: the model says the step ends `consumed + cost` after the bubble began; if the
        // host is later than that, the step must still end before the declared end of the bubble
        const uint64_t consumed = (uint64_t)(total - remaining);
        const uint64_t now = now_ns();
        const uint64_t start_est = now > t_begin + consumed ? now : t_begin + consumed;
        if (start_est + cost > t_begin + len) {
            std::lock_guard<std::mutex> lk(c->mu);
            fr_event ev{};
            ev.kind = FR_EV_MISS; ev.bubble = index; ev.run = st.run; ev.segment = st.segment;
            ev.tile0 = st.tile0; ev.tile1 = st.tile1; ev.modelled_ns = cost; ev.work_units = st.work_units;
            ev.t_host_ns = now;
            log_push(c, ev);
            t->prog.deadline_misses++;
            break;
        }
        if (timed) {
            // bound the number of steps enqueued ahead of the GPU
            bool left = false;
            for (;;) {
                size_t inflight;
                {
                    std::lock_guard<std::mutex> lk(c->mu);
                    resolve_timings(c, false);
                    inflight = c->pending.size();
                }
                if (inflight < max_inflight) break;
                if (stop_now()) { left = true; break; }
                cpu_relax();
            }
            if (left) break;
        }
        if (timed && group_n == 0) {
            // a new group begins where the previous one ended, or, at the head of the chain, at an event of its own
            bool chain_head = false;
            {
                std::lock_guard<std::mutex> lk(c->mu);
                if (c->chain_tail) group_begin = c->chain_tail;
                else { group_begin = event_get(c); chain_head = true; }
            }
            if (chain_head && group_begin) (void)hipEventRecord(group_begin, c->side);
        }
        if (gated) {
            st.gate = c->gate;
            st.gate_slot = (uint32_t)c->gate_steps.size();
            const double need = (double)scaled * c->ticks_per_ns;
            st.gate_need_ticks = need < 4.0e9 ? (uint32_t)need : 4000000000u;
            // the heaviest tile's time alone, scaled like the step's cost
            const double tile = st.modelled_ns ? (double)st.gate_tile * ((double)scaled / (double)st.modelled_ns) * c->ticks_per_ns : 0.0;
            st.gate_tile = tile < 4.0e9 ? (uint32_t)tile : 4000000000u;
        }
        c->in_callback.store(now_ns(), std::memory_order_release);
        rc = t->ops.run_step(t->user, (void*)c->side, &st);
        c->in_callback.store(0, std::memory_order_release);
        {
            std::lock_guard<std::mutex> lk(c->mu);
            fr_event ev{};
            ev.kind = FR_EV_CHUNK; ev.bubble = index; ev.run = st.run; ev.segment = st.segment;
            ev.tile0 = st.tile0; ev.tile1 = st.tile1; ev.modelled_ns = cost; ev.work_units = st.work_units;
            ev.t_host_ns = now;
            group_last_seq = log_push(c, ev);
            t->prog.steps++;
            t->prog.work_units_done += st.work_units;
            t->prog.ns_modelled += cost;
            if (st.completes_run) t->prog.runs_completed++;
            if (!used) { used = true; t->prog.bubbles_used++; }
        }
        if (gated) { c->gate_steps.push_back(st); c->gate_bubble.push_back(index); c->gate_seq.push_back(group_last_seq); }
        if (timed) {
            group_n++; group_mask |= 1u << (st.cost_class & 7); group_modelled += st.modelled_ns;
            if (group_n >= group_size) close_group();
        }
        if (rc != FR_OK) { fail = rc; break; }
        if (c->kill_current.load(std::memory_order_acquire)) break;
        remaining -= (int64_t)cost;
    }
    if (timed && group_n) close_group();
    if (gated) c->gate_pending.store(!c->gate_steps.empty());
    if (used && !c->host_only && c->tail_event) c->tail_armed = hipEventRecord(c->tail_event, c->side) == hipSuccess;
    std::lock_guard<std::mutex> lk(c->mu);
    if (c->chain_tail) {
        // close the chain: nobody will begin at its tail any more
        bool unresolved = false;
        for (const PendingTiming& p : c->pending) unresolved |= (p.end == c->chain_tail);
        if (!unresolved) c->free_events.push_back(c->chain_tail);
        c->chain_tail = nullptr;
    }
    if (fail != FR_OK) stop_task_locked(c, t, fail);
    else if (c->kill_current.exchange(false)) {
        t->prog.killed = 1;
        stop_task_locked(c, t, FR_ERR_OVERRUN);
    } else if (finished && !c->queue.empty()) stop_task_locked(c, t, FR_OK);   // done: the worker moves on to the next task
    else if (t->state == FR_RUNNING) t->state = FR_PAUSED;   // PauseSideTask()
    if (t->state == FR_STOPPED) promote_locked(c);
}

void worker_main(fr_ctx* c)
{
    if (!c->host_only) (void)hipSetDevice(c->cfg.device_id);
    uint64_t seen = 0;
    uint32_t idle_spins = 0;
    while (!c->quit.load(std::memory_order_acquire)) {
        const uint64_t seq = c->bubble_seq.load(std::memory_order_acquire);
        if (seq == seen && c->gate_pending.load() && c->tail_armed && hipEventQuery(c->tail_event) == hipSuccess) {
            std::lock_guard<std::mutex> wl(c->work_mu);      // the bubble's work has drained: read its verdicts
            Task* t;
            { std::lock_guard<std::mutex> lk(c->mu); t = c->task; }
            gate_settle(c, t);
        }
        if (seq == seen) {
            // Spin while a live task may be handed a bubble at any moment; back off otherwise.
            if (++idle_spins > 20000) {
                bool live;
                {
                    std::lock_guard<std::mutex> lk(c->mu);
                    live = c->task && c->task->state != FR_STOPPED;
                    if (live && !c->pending.empty()) resolve_timings(c, false);
                }
                if (!live) std::this_thread::sleep_for(std::chrono::microseconds(200));
                idle_spins = 0;
            } else cpu_relax();
            continue;
        }
        idle_spins = 0;
        seen = seq;
        uint64_t t_begin, len, served = seq;
        uint32_t index;
        for (;;) {
            t_begin = c->cur_begin.load(std::memory_order_relaxed);
            len = c->cur_len.load(std::memory_order_relaxed);
            index = c->cur_index.load(std::memory_order_relaxed);
            const uint64_t again = c->bubble_seq.load(std::memory_order_acquire);
            if (again == served) break;
            served = again;
        }
        seen = served;
        c->tail_armed = false;
        {
            std::lock_guard<std::mutex> wl(c->work_mu);
            serve_bubble(c, served, t_begin, len, index);
        }
        c->ack_seq.store(served, std::memory_order_release);
    }
}

// ctx->mu held; stage thread, the bubble in question is the one being closed.
void note_overrun(fr_ctx* c)
{
    if (c->task) c->task->prog.overruns++;
    fr_event ev{};
    ev.kind = FR_EV_OVERRUN; ev.bubble = c->cur_index.load(std::memory_order_relaxed); ev.t_host_ns = now_ns();
    log_push(c, ev);
}

// Allocates the gate and measures how the GPU's wall clock relates to the host's: a one-thread kernel stores
// wall_clock64(), the host notes its own clock before the launch and after the wait; the tightest of a few
// such windows gives the offset (good to a few microseconds, which guard_ns must cover).
// `rounds` windows on an idle side stream, the first `skip` of them not counted; the tightest one is taken if it is
// no wider than `at_most`.
int gate_read_clock(fr_ctx* c, int rounds, int skip, uint64_t at_most)
{
    uint64_t best_window = ~0ull;
    int64_t best_offset = 0;
    for (int i = 0; i < rounds; ++i) {
        const uint64_t t0 = now_ns();
        hipLaunchKernelGGL(k_gate_clock, dim3(1), dim3(1), 0, c->side, c->gate);
        if (hipStreamSynchronize(c->side) != hipSuccess) return FR_ERR_HIP;
        const uint64_t t1 = now_ns();
        unsigned long long ticks = 0;
        if (hipMemcpy(&ticks, &c->gate->deadline_ticks, sizeof(ticks), hipMemcpyDeviceToHost) != hipSuccess) return FR_ERR_HIP;
        if (i >= skip && t1 - t0 < best_window) {
            best_window = t1 - t0;
            best_offset = (int64_t)((double)ticks / c->ticks_per_ns) - (int64_t)(t0 + (t1 - t0) / 2);
        }
    }
    if (best_window <= at_most) {
        c->gpu_minus_host_ns = best_offset;
        c->clock_window_ns = best_window;
        c->clock_read_ns = now_ns();
    }
    return FR_OK;
}

int gate_setup(fr_ctx* c)
{
    int khz = 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, c->cfg.device_id) != hipSuccess || khz <= 0) return FR_ERR_HIP;
    c->ticks_per_ns = (double)khz * 1.0e-6;
    if (hipMalloc(reinterpret_cast<void**>(&c->gate), sizeof(fr_gate)) != hipSuccess) { c->gate = nullptr; return FR_ERR_HIP; }
    if (hipMemset(c->gate, 0, sizeof(fr_gate)) != hipSuccess) return FR_ERR_HIP;
    return gate_read_clock(c, 12, 2, ~0ull);                    // (the first launches pay one-time costs)
}

// The two clocks drift apart (some tens of microseconds a second were seen), so the reading is renewed now and then,
// at the start of a bubble, when the side stream is idle anyway: three windows, about 50 us, four times a second at
// most; a reading from a window much wider than the first one's (something held the stream up) is not taken.
constexpr uint64_t kClockRereadNs = 250000000;
void gate_refresh_clock(fr_ctx* c)
{
    if (now_ns() - c->clock_read_ns < kClockRereadNs) return;
    const uint64_t before = c->clock_read_ns;
    (void)gate_read_clock(c, 3, 0, 2 * c->clock_window_ns + 2000);
    if (c->clock_read_ns == before) c->clock_read_ns = now_ns() - kClockRereadNs / 2;      // not taken: try again sooner
}

// How long fr_bubble_end waits for a step callback that is still running after the bubble's end.
constexpr uint64_t kCallbackPatienceNs = 200000;
// How long fr_bubble_end re-asks whether the marker behind the bubble's last step has retired.
constexpr uint64_t kTailPatienceNs = 20000;

// Stage thread, between bubbles or at a bubble's edge: has the work that was late at an earlier bubble end
// finished meanwhile?  If not and the grace period is over, ask the worker to stop the task.
void enforce_check(fr_ctx* c)
{
    if (!c->enforce_armed) return;
    bool still_late;
    if (c->enforce_gpu) still_late = c->tail_event && hipEventQuery(c->tail_event) == hipErrorNotReady;
    else if (c->enforce_callback == 1) still_late = c->in_init.load(std::memory_order_acquire);
    else still_late = c->in_callback.load(std::memory_order_acquire) == c->enforce_callback;
    if (!still_late) { c->enforce_armed = false; return; }
    if (now_ns() < c->enforce_deadline) return;
    c->kill_current.store(true, std::memory_order_release);
    c->enforce_armed = false;
}

}  // namespace

// ------------------------------------------------------------------ allocator
void fr_alloc_reset(fr_alloc* a, uint64_t limit, bool host_only, int device)
{
    a->limit = limit; a->used = 0; a->oom = false; a->host_only = host_only; a->device = device;
    a->hip_error = 0; a->peak = 0; a->blocks.clear();
}

void fr_alloc_release(fr_alloc* a)
{
    for (const fr_alloc::Block& b : a->blocks) {
        if (a->host_only) std::free(b.ptr);
        else (void)hipFree(b.ptr);
    }
    a->blocks.clear();
    a->used = 0;
}

extern "C" {

uint64_t fr_now_ns(void) { return now_ns(); }

void* fr_alloc_device(fr_alloc* a, size_t bytes)
{
    if (!a || a->oom) return nullptr;
    const uint64_t rounded = ((uint64_t)bytes + 255) & ~255ull;
    if (rounded > a->limit || a->used > a->limit - rounded) { a->oom = true; return nullptr; }
    void* p = nullptr;
    if (a->host_only) {
        p = std::aligned_alloc(256, rounded ? rounded : 256);
        if (!p) { a->oom = true; return nullptr; }
    } else {
        hipError_t e = hipMalloc(&p, rounded ? rounded : 256);
        if (e != hipSuccess) { a->hip_error = (int)e; a->oom = true; return nullptr; }
    }
    a->blocks.push_back({p, rounded});
    a->used += rounded;
    if (a->used > a->peak) a->peak = a->used;
    return p;
}

int fr_alloc_free(fr_alloc* a, void* p)
{
    if (!a || !p) return FR_ERR_ARG;
    for (size_t i = 0; i < a->blocks.size(); ++i) {
        if (a->blocks[i].ptr != p) continue;
        if (a->host_only) std::free(p);
        else (void)hipFree(p);
        a->used -= a->blocks[i].bytes;
        a->blocks.erase(a->blocks.begin() + (long)i);
        return FR_OK;
    }
    return FR_ERR_ARG;
}

int fr_alloc_charge(fr_alloc* a, size_t bytes)
{
    if (!a) return FR_ERR_ARG;
    if (a->oom) return FR_ERR_OOM;
    if ((uint64_t)bytes > a->limit || a->used > a->limit - (uint64_t)bytes) { a->oom = true; return FR_ERR_OOM; }
    a->used += bytes;
    if (a->used > a->peak) a->peak = a->used;
    return FR_OK;
}

uint64_t fr_alloc_used(const fr_alloc* a) { return a ? a->used : 0; }
uint64_t fr_alloc_peak(const fr_alloc* a) { return a ? a->peak : 0; }

// ------------------------------------------------------------------ context
int fr_create(const fr_config* cfg, fr_ctx** out)
{
    if (!cfg || !out) return FR_ERR_ARG;
    if (cfg->cu_count > 256) return FR_ERR_ARG;
    fr_ctx* c = new (std::nothrow) fr_ctx();
    if (!c) return FR_ERR_ARG;
    c->cfg = *cfg;
    c->host_only = cfg->device_id < 0;
    c->log.resize(cfg->event_log_capacity ? cfg->event_log_capacity : 65536);
    if (!c->host_only) {
        int n = 0;
        hipError_t e = hipGetDeviceCount(&n);
        if (e != hipSuccess || cfg->device_id >= n) { c->hip_error = (int)e; delete c; return e != hipSuccess ? FR_ERR_HIP : FR_ERR_ARG; }
        e = hipSetDevice(cfg->device_id);
        if (e != hipSuccess) { delete c; return FR_ERR_HIP; }
        uint32_t mask[8] = {0};
        bool masked = false;
        if (cfg->cu_count > 0 && cfg->cu_count < 256) {
            for (uint32_t i = 0; i < cfg->cu_count; ++i) mask[i / 32] |= 1u << (i % 32);
            masked = true;
        } else if (cfg->cu_count == 0) {
            for (int i = 0; i < 8; ++i) { mask[i] = cfg->cu_mask[i]; masked |= mask[i] != 0; }
        }
        if (masked) {
            // a mask that leaves out no compute unit asks for what a plain stream is
            int cus = 0, set = 0;
            for (uint32_t w : mask) set += __builtin_popcount(w);
            if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, cfg->device_id) == hipSuccess && cus > 0 && set >= cus)
                masked = false;
        }
        // Both stream kinds keep the default priority.
        if (masked) e = hipExtStreamCreateWithCUMask(&c->side, 8, mask);
        else e = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking);
        if (e != hipSuccess) { delete c; return FR_ERR_HIP; }
        e = hipEventCreateWithFlags(&c->tail_event, hipEventDisableTiming);
        if (e != hipSuccess) { (void)hipStreamDestroy(c->side); delete c; return FR_ERR_HIP; }
        if (cfg->device_gate && gate_setup(c) != FR_OK) {
            (void)hipEventDestroy(c->tail_event); (void)hipStreamDestroy(c->side);
            if (c->gate) (void)hipFree(c->gate);
            delete c;
            return FR_ERR_HIP;
        }
    }
    c->worker = std::thread(worker_main, c);
    *out = c;
    return FR_OK;
}

int fr_destroy(fr_ctx* c)
{
    if (!c) return FR_ERR_ARG;
    c->abort_steps.store(true);
    c->end_requested.store(true);
    c->quit.store(true, std::memory_order_release);
    if (c->worker.joinable()) c->worker.join();
    {
        std::lock_guard<std::mutex> lk(c->mu);
        if (c->task) stop_task_locked(c, c->task, FR_OK);
        c->task = nullptr;
        c->queue.clear();
        for (Task* t : c->tasks) delete t;
        c->tasks.clear();
        resolve_timings(c, true);
        for (hipEvent_t e : c->free_events) (void)hipEventDestroy(e);
        c->free_events.clear();
    }
    if (c->side) { (void)hipStreamSynchronize(c->side); (void)hipStreamDestroy(c->side); }
    if (c->tail_event) (void)hipEventDestroy(c->tail_event);
    if (c->gate) (void)hipFree(c->gate);
    delete c;
    return FR_OK;
}

int fr_side_stream(fr_ctx* c, void** out)
{
    if (!c || !out) return FR_ERR_ARG;
    *out = (void*)c->side;
    return FR_OK;
}

int fr_last_hip_error(fr_ctx* c) { return c ? c->hip_error : 0; }

// ------------------------------------------------------------------ task
int fr_task_register(fr_ctx* c, const fr_task_ops* ops, void* user, const fr_task_profile* prof, fr_task_id* id_out)
{
    if (!c || !ops || !prof || !id_out || !ops->plan_step || !ops->run_step) return FR_ERR_ARG;
    // Algorithm 1 with a single worker: the worker qualifies only if its free memory exceeds the task's need.
    if (!(c->cfg.mem_available_bytes > prof->mem_limit_bytes)) return FR_ERR_NOMEM;   // RejectSideTask()
    std::lock_guard<std::mutex> wl(c->work_mu);
    std::lock_guard<std::mutex> lk(c->mu);
    Task* t = new (std::nothrow) Task();
    if (!t) return FR_ERR_ARG;
    t->ops = *ops; t->user = user; t->prof = *prof; t->id = c->next_id++;
    fr_alloc_reset(&t->alloc, prof->mem_limit_bytes, c->host_only, c->cfg.device_id);
    t->state = FR_SUBMITTED;
    c->tasks.push_back(t);
    c->queue.push_back(t);                   // Algorithm 1: AddToQueue
    promote_locked(c);                       // Algorithm 2: becomes current at once if the worker has no live task
    if (t->state == FR_STOPPED) {            // its create() failed
        const int rc = t->last_error;
        c->tasks.pop_back();
        delete t;
        return rc;
    }
    *id_out = t->id;
    return FR_OK;
}

int fr_task_stop(fr_ctx* c, fr_task_id id)
{
    if (!c) return FR_ERR_ARG;
    c->abort_steps.store(true);
    std::lock_guard<std::mutex> wl(c->work_mu);     // the worker is outside every callback now
    c->abort_steps.store(false);
    std::lock_guard<std::mutex> lk(c->mu);
    Task* t = find_task(c, id);
    if (!t) return FR_ERR_ARG;
    if (t->state == FR_STOPPED) return FR_ERR_STATE;
    if (t->state == FR_SUBMITTED) {          // still waiting in the queue: it just leaves it
        for (size_t i = 0; i < c->queue.size(); ++i)
            if (c->queue[i] == t) { c->queue.erase(c->queue.begin() + (long)i); break; }
        t->state = FR_STOPPED;
        return FR_OK;
    }
    stop_task_locked(c, t, FR_OK);
    promote_locked(c);
    return FR_OK;
}

int fr_bubble_begin(fr_ctx* c, uint64_t t_begin_ns, uint64_t duration_ns)
{
    if (!c) return FR_ERR_ARG;
    if (c->bubble_open) return FR_ERR_STATE;
    enforce_check(c);
    c->bubble_open = true;
    c->cur_begin.store(t_begin_ns, std::memory_order_relaxed);
    c->cur_len.store(duration_ns, std::memory_order_relaxed);
    c->cur_index.store((uint32_t)c->bubbles_total++, std::memory_order_relaxed);
    c->end_requested.store(false, std::memory_order_release);
    c->bubble_seq.fetch_add(1, std::memory_order_release);
    return FR_OK;
}

int fr_bubble_end(fr_ctx* c)
{
    if (!c) return FR_ERR_ARG;
    if (!c->bubble_open) return FR_ERR_STATE;
    enforce_check(c);
    c->end_requested.store(true, std::memory_order_release);
    const uint64_t seq = c->bubble_seq.load(std::memory_order_acquire);
    while (c->ack_seq.load(std::memory_order_acquire) != seq) {              // worker enqueues nothing more
        // A callback that outlives the bubble does not hold the stage up: the call returns at once for
        // InitSideTask (known to be long) and after kCallbackPatience for a step callback, and the work goes on
        // beside the stage's next operation until it returns or the grace period runs out.
        const bool init_late = c->in_init.load(std::memory_order_acquire);
        const uint64_t cb = c->in_callback.load(std::memory_order_acquire);
        const uint64_t now = now_ns();
        if (init_late || (cb && now > cb + kCallbackPatienceNs && now > c->cur_begin.load(std::memory_order_relaxed) + c->cur_len.load(std::memory_order_relaxed))) {
            c->bubble_open = false;
            if (c->cfg.grace_ns && !c->enforce_armed) {
                c->enforce_armed = true; c->enforce_gpu = false;
                c->enforce_callback = init_late ? 1 : cb;
                c->enforce_deadline = now + c->cfg.grace_ns;
            }
            std::lock_guard<std::mutex> lk(c->mu);
            note_overrun(c);
            return FR_ERR_OVERRUN;
        }
        cpu_relax();
    }
    c->bubble_open = false;
    if (c->host_only || !c->tail_armed) return FR_OK;     // nothing was enqueued for this bubble
    // The marker behind the bubble's last step may have been submitted microseconds ago and needs a moment to
    // retire even on an idle stream, so "not ready" is only believed if it persists for kTailPatienceNs.
    hipError_t q = hipEventQuery(c->tail_event);
    for (const uint64_t t0 = now_ns(); q == hipErrorNotReady && now_ns() - t0 < kTailPatienceNs;) {
        cpu_relax();
        q = hipEventQuery(c->tail_event);
    }
    if (q == hipErrorNotReady) {
        if (c->cfg.grace_ns && !c->enforce_armed) {
            c->enforce_armed = true; c->enforce_gpu = true;
            c->enforce_deadline = now_ns() + c->cfg.grace_ns;
        }
        std::lock_guard<std::mutex> lk(c->mu);
        note_overrun(c);
        return FR_ERR_OVERRUN;
    }
    if (q != hipSuccess) { c->hip_error = (int)q; return FR_ERR_HIP; }
    return FR_OK;
}

int fr_query_progress(fr_ctx* c, fr_task_id id, fr_progress* out)
{
    if (!c || !out) return FR_ERR_ARG;
    std::lock_guard<std::mutex> lk(c->mu);
    Task* t = find_task(c, id);
    if (!t) return FR_ERR_ARG;
    if (!c->host_only) resolve_timings(c, false);
    *out = t->prog;
    out->state = t->state;
    out->last_error = t->last_error;
    if (t->state != FR_STOPPED) out->mem_used_bytes = t->alloc.used;
    return FR_OK;
}

int fr_event_log(fr_ctx* c, fr_event* buf, size_t cap, size_t* n_out)
{
    if (!c || !n_out || (!buf && cap)) return FR_ERR_ARG;
    std::lock_guard<std::mutex> lk(c->mu);
    if (!c->host_only) resolve_timings(c, false);
    const size_t n = c->log_count < cap ? c->log_count : cap;
    for (size_t i = 0; i < n; ++i) buf[i] = c->log[(c->log_head + i) % c->log.size()];
    *n_out = n;
    return FR_OK;
}

int fr_event_log_clear(fr_ctx* c)
{
    if (!c) return FR_ERR_ARG;
    std::lock_guard<std::mutex> lk(c->mu);
    if (!c->host_only) resolve_timings(c, true);
    c->log_first_seq += c->log_count;
    c->log_head = 0;
    c->log_count = 0;
    return FR_OK;
}

uint32_t fr_cost_scale_next(uint32_t scale_ppm, uint64_t modelled_ns, uint64_t measured_ns)
{
    if (scale_ppm < kScaleMin) scale_ppm = kScaleMin;
    if (scale_ppm > kScaleMax) scale_ppm = kScaleMax;
    if (modelled_ns == 0) return scale_ppm;
    unsigned __int128 r128 = (unsigned __int128)measured_ns * kScaleOne / modelled_ns;
    uint32_t r = r128 > kScaleMax ? kScaleMax : (uint32_t)r128;
    if (r < kScaleMin) r = kScaleMin;
    if (r >= scale_ppm) return r > 2 * scale_ppm ? 2 * scale_ppm : r;     // one late step at most doubles the scale
    return scale_ppm - (scale_ppm - r) / 8;
}

int fr_cost_scales(fr_ctx* c, uint32_t* out)
{
    if (!c || !out) return FR_ERR_ARG;
    std::lock_guard<std::mutex> lk(c->mu);
    if (!c->host_only) resolve_timings(c, false);
    if (c->pending.empty()) apply_totals(c);
    for (int i = 0; i < 8; ++i) out[i] = c->cost_scale[i];
    return FR_OK;
}

int fr_chunk_fit(const uint64_t* prefix, uint32_t n_tiles, uint32_t tile0, uint64_t budget_ns,
                 uint64_t launch_cost_ns, uint32_t* n_fit)
{
    if (!prefix || !n_fit || tile0 > n_tiles) return FR_ERR_ARG;
    *n_fit = 0;
    if (budget_ns < launch_cost_ns) return FR_OK;
    const uint64_t room = budget_ns - launch_cost_ns;
    const uint64_t base = prefix[tile0];
    // largest index hi in [tile0, n_tiles] with prefix[hi] - base <= room
    uint32_t lo = tile0, hi = n_tiles;
    while (lo < hi) {
        const uint32_t mid = lo + (hi - lo + 1) / 2;
        if (prefix[mid] - base <= room) lo = mid;
        else hi = mid - 1;
    }
    *n_fit = lo - tile0;
    return FR_OK;
}

}  // extern "C"
