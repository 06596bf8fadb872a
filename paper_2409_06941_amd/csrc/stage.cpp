// Stage emulator: one stage of a pipeline-parallel epoch with the waits the other stages impose.
//
// Follows the paper's description of pipeline training (Section 2.1: every micro-batch has a forward and a
// backward pass on every stage; a stage passes its output on and moves to its next operation at once) and of
// bubbles as idle periods caused by unsatisfied FP/BP dependencies (Section 2.1, Section 2.2.1).  Bubbles are
// reported to the runtime at the points the paper instruments (Section 4.6): before the first and after the
// last operation of an epoch, and wherever the stage waits inside the epoch.
//
// Ideal timing model: p stages, m micro-batches, every FP lasts f and every BP lasts b on every stage, zero
// hand-over time.  The finish time of each operation is the longest path through the dependency graph
// (previous operation of the same stage; FP of the previous stage / BP of the next stage; on the last stage
// the BP follows its own FP), evaluated with memoised recursion.

#include <time.h>

#include <algorithm>
#include <new>
#include <thread>

#include "common.h"

namespace {

struct OpRef { int kind; int mb; int chunk; };   // kind 0 = FP, 1 = BP; chunk: model chunk (interleaved schedule)

// Serial order of stage s.  GPipe: all forwards then all backwards.  1F1B: min(p - 1 - s, m) warm-up forwards,
// then one forward / one backward alternately, then the backwards that are left.  Interleaved 1F1B (Narayanan et
// al. 2021, one of the bubble-reducing schedules the paper's Sections 1 and 2.2.2 refer to): the stage holds v model
// chunks, chunk c being virtual stage c p + s; with n = m v operations of each kind, min(n, 2 (p - 1 - s) + (v - 1) p)
// warm-up forwards, then pairs, then the backwards that are left; the k-th forward is chunk (k mod p v) div p of
// micro-batch (k div p v) p + k mod p, the k-th backward the same micro-batch of chunk v - 1 - (k mod p v) div p.
std::vector<OpRef> order_of(int schedule, int p, int m, int v, int s)
{
    std::vector<OpRef> o;
    o.reserve(2 * (size_t)m * (size_t)v);
    if (schedule == FR_SCHED_GPIPE) {
        for (int j = 0; j < m; ++j) o.push_back({0, j, 0});
        for (int j = 0; j < m; ++j) o.push_back({1, j, 0});
        return o;
    }
    if (schedule == FR_SCHED_INTERLEAVED) {
        const int n = m * v, pv = p * v;
        auto fwd = [&](int k) { return OpRef{0, (k / pv) * p + k % p, (k % pv) / p}; };
        auto bwd = [&](int k) { return OpRef{1, (k / pv) * p + k % p, v - 1 - (k % pv) / p}; };
        const int warm = std::min(n, 2 * (p - 1 - s) + (v - 1) * p);
        int f = 0, b = 0;
        for (; f < warm; ++f) o.push_back(fwd(f));
        while (b < n) {
            if (f < n) o.push_back(fwd(f++));
            o.push_back(bwd(b++));
        }
        return o;
    }
    const int warm = std::min(p - 1 - s, m);
    int f = 0, b = 0;
    for (; f < warm; ++f) o.push_back({0, f, 0});
    while (b < m) {
        if (f < m) o.push_back({0, f++, 0});
        o.push_back({1, b++, 0});
    }
    return o;
}

// The dependency graph runs over virtual stages vs = chunk * p + stage (vs = stage when there is one chunk): FP of
// vs needs FP of vs - 1, BP of vs needs BP of vs + 1, and on the last virtual stage the BP needs its own FP.
struct IdealSchedule {
    int p, m, v;
    uint64_t f, b;
    std::vector<std::vector<OpRef>> order;          // [stage][slot]
    std::vector<std::vector<int>> slot_of[2];       // [kind][stage][chunk * m + mb] -> slot
    std::vector<std::vector<int64_t>> finish;       // [stage][slot], -1 = not yet known

    int64_t finish_vs(int kind, int vs, int mb) { return finish_of(vs % p, slot_of[kind][vs % p][(vs / p) * m + mb]); }

    int64_t finish_of(int s, int slot)
    {
        int64_t& memo = finish[s][slot];
        if (memo >= 0) return memo;
        const OpRef op = order[s][slot];
        const int vs = op.chunk * p + s;
        int64_t ready = slot > 0 ? finish_of(s, slot - 1) : 0;
        if (op.kind == 0) {
            if (vs > 0) ready = std::max(ready, finish_vs(0, vs - 1, op.mb));
        } else if (vs == v * p - 1) {
            ready = std::max(ready, finish_vs(0, vs, op.mb));
        } else {
            ready = std::max(ready, finish_vs(1, vs + 1, op.mb));
        }
        memo = ready + (int64_t)(op.kind == 0 ? f : b);
        return memo;
    }
};

uint64_t clock_ns()
{
    timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return (uint64_t)ts.tv_sec * 1000000000ull + (uint64_t)ts.tv_nsec;
}

void wait_until(uint64_t t_ns)
{
    // sleep for the bulk of the wait, spin for the last stretch
    for (;;) {
        const uint64_t now = clock_ns();
        if (now >= t_ns) return;
        const uint64_t left = t_ns - now;
        if (left > 200000) std::this_thread::sleep_for(std::chrono::nanoseconds(left - 150000));
        else __builtin_ia32_pause();
    }
}

}  // namespace

struct fr_stage {
    fr_stage_desc d{};
    fr_load* load = nullptr;
    hipStream_t stream = nullptr;
    bool own_stream = false;
    std::vector<fr_stage_op> ops;
    uint64_t epoch_ns = 0, tail_ns = 0;
    std::vector<uint64_t> op_ns;            // measured burst times of the latest epoch, one per operation
    hipStream_t filler_stream = nullptr;    // fr_stage_set_filler
    uint32_t filler_workgroups = 0;
    uint64_t filler_guard_ns = 0;
    int wall_clock_khz = 100000;
};

extern "C" {

int fr_stage_make(const fr_stage_desc* d, fr_load* load, void* stage_stream, fr_stage** out)
{
    if (!d || !out) return FR_ERR_ARG;
    if (d->schedule != FR_SCHED_1F1B && d->schedule != FR_SCHED_GPIPE && d->schedule != FR_SCHED_INTERLEAVED) return FR_ERR_ARG;
    if (d->p < 1 || d->m < 1 || d->stage < 0 || d->stage >= d->p || d->f_ns == 0 || d->b_ns == 0) return FR_ERR_ARG;
    if (d->p > 1024 || d->m > 4096) return FR_ERR_ARG;   // keeps the recursion shallow
    const int v = d->schedule == FR_SCHED_INTERLEAVED ? d->chunks : 1;
    if (v < 1 || v > 64 || (d->schedule == FR_SCHED_INTERLEAVED && d->m % d->p != 0)) return FR_ERR_ARG;
    if (d->schedule != FR_SCHED_INTERLEAVED && d->chunks > 1) return FR_ERR_ARG;
    fr_stage* s = new (std::nothrow) fr_stage();
    if (!s) return FR_ERR_ARG;
    s->d = *d;
    s->load = load;
    s->stream = (hipStream_t)stage_stream;

    IdealSchedule is;
    is.p = d->p; is.m = d->m; is.v = v; is.f = d->f_ns; is.b = d->b_ns;
    is.order.resize(d->p);
    is.slot_of[0].assign(d->p, std::vector<int>((size_t)d->m * v, -1));
    is.slot_of[1].assign(d->p, std::vector<int>((size_t)d->m * v, -1));
    is.finish.resize(d->p);
    for (int st = 0; st < d->p; ++st) {
        is.order[st] = order_of(d->schedule, d->p, d->m, v, st);
        is.finish[st].assign(is.order[st].size(), -1);
        for (size_t k = 0; k < is.order[st].size(); ++k) {
            const OpRef& op = is.order[st][k];
            is.slot_of[op.kind][st][(size_t)op.chunk * d->m + op.mb] = (int)k;
        }
    }
    int64_t epoch = 0;
    for (int st = 0; st < d->p; ++st) epoch = std::max(epoch, is.finish_of(st, (int)is.order[st].size() - 1));
    const auto& mine = is.order[d->stage];
    int64_t prev_end = 0;
    for (size_t k = 0; k < mine.size(); ++k) {
        const int64_t end = is.finish_of(d->stage, (int)k);
        const int64_t start = end - (int64_t)(mine[k].kind == 0 ? d->f_ns : d->b_ns);
        fr_stage_op op{};
        op.kind = mine[k].kind; op.microbatch = mine[k].mb; op.chunk = mine[k].chunk;
        op.start_ns = (uint64_t)start; op.end_ns = (uint64_t)end;
        op.bubble_before_ns = (uint64_t)(start - prev_end);
        s->ops.push_back(op);
        prev_end = end;
    }
    s->epoch_ns = (uint64_t)epoch;
    s->tail_ns = (uint64_t)(epoch - prev_end);
    *out = s;
    return FR_OK;
}

int fr_stage_destroy(fr_stage* s)
{
    if (!s) return FR_ERR_ARG;
    delete s;
    return FR_OK;
}

int fr_stage_ops(fr_stage* s, fr_stage_op* buf, size_t cap, size_t* n_out, uint64_t* epoch_ns_out, uint64_t* tail_out)
{
    if (!s || !n_out || (!buf && cap)) return FR_ERR_ARG;
    const size_t n = std::min(cap, s->ops.size());
    for (size_t i = 0; i < n; ++i) buf[i] = s->ops[i];
    *n_out = s->ops.size();
    if (epoch_ns_out) *epoch_ns_out = s->epoch_ns;
    if (tail_out) *tail_out = s->tail_ns;
    return FR_OK;
}

int fr_stage_set_filler(fr_stage* s, void* stream, uint32_t workgroups, uint64_t guard_ns)
{
    if (!s) return FR_ERR_ARG;
    if (workgroups > 65536) return FR_ERR_ARG;
    int device = 0, khz = 0;
    if (workgroups && (hipGetDevice(&device) != hipSuccess ||
                       hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, device) != hipSuccess || khz <= 0))
        return FR_ERR_HIP;
    if (workgroups) s->wall_clock_khz = khz;
    s->filler_stream = (hipStream_t)stream;
    s->filler_workgroups = workgroups;
    s->filler_guard_ns = guard_ns;
    return FR_OK;
}

int fr_stage_op_times(fr_stage* s, uint64_t* ns_host, size_t cap, size_t* n_out)
{
    if (!s || !n_out || (!ns_host && cap)) return FR_ERR_ARG;
    const size_t n = std::min(cap, s->op_ns.size());
    for (size_t i = 0; i < n; ++i) ns_host[i] = s->op_ns[i];
    *n_out = s->op_ns.size();
    return FR_OK;
}

int fr_stage_run_epoch(fr_stage* s, fr_ctx* ctx, fr_epoch_result* out)
{
    if (!s || !out || !s->load) return FR_ERR_ARG;
    fr_epoch_result r{};
    int hip_err = 0;
    s->op_ns.clear();
    auto bubble = [&](uint64_t len) -> int {
        const uint64_t tb = clock_ns();
        if (ctx) {
            int rc = fr_bubble_begin(ctx, tb, len);
            if (rc != FR_OK) return rc;
        } else if (s->filler_workgroups && len > s->filler_guard_ns) {
            int rc = fr_alufill_launch(len - s->filler_guard_ns, s->wall_clock_khz, s->filler_workgroups, s->filler_stream);
            if (rc != FR_OK) return rc;
        }
        wait_until(tb + len);          // the other stages' work, as a timed wait
        if (!ctx && s->filler_workgroups && len > s->filler_guard_ns) FR_HIP_TRY(hipStreamSynchronize(s->filler_stream), hip_err);
        if (ctx) {
            int rc = fr_bubble_end(ctx);
            if (rc == FR_ERR_OVERRUN) r.overruns++;
            else if (rc != FR_OK) return rc;
        }
        r.bubble_ns += len;
        r.n_bubbles++;
        return FR_OK;
    };
    const uint64_t t0 = clock_ns();
    for (const fr_stage_op& op : s->ops) {
        if (op.bubble_before_ns) {
            int rc = bubble(op.bubble_before_ns);
            if (rc != FR_OK) return rc;
        }
        const uint64_t a = clock_ns();
        const int parts = s->d.schedule == FR_SCHED_INTERLEAVED ? s->d.chunks : 1;
        int rc = fr_load_part(s->load, (void*)s->stream, op.kind, op.chunk, parts);
        if (rc != FR_OK) return rc;
        FR_HIP_TRY(hipStreamSynchronize(s->stream), hip_err);
        const uint64_t took = clock_ns() - a;
        r.busy_ns += took;
        s->op_ns.push_back(took);
        r.n_ops++;
    }
    if (s->tail_ns) {
        int rc = bubble(s->tail_ns);
        if (rc != FR_OK) return rc;
    }
    r.epoch_ns = clock_ns() - t0;
    *out = r;
    return FR_OK;
}

}  // extern "C"
