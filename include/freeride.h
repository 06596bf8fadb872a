/*
 * freeride.h -- C ABI of the bubble-harvesting runtime for one pipeline stage on one GPU.
 *
 * The library serves one GPU "side task" inside the idle windows (bubbles) of a pipeline-parallel training
 * stage, after FreeRide (arXiv 2409.06941):
 *   - the side task is a state machine with the states SUBMITTED, CREATED, PAUSED, RUNNING, STOPPED and the
 *     transitions Create / Init / Start / Pause / RunNextStep / Stop (Section 4.1, Figure 3);
 *   - the training system reports every bubble (start time, duration) to the manager (Section 3.2, Section 4.6),
 *     which initialises or starts the current task when a bubble begins and pauses it when the bubble ends
 *     (Section 4.4, Algorithm 2);
 *   - before every step the task checks that the time left in the bubble is enough for that step
 *     (program-directed time limit, Section 4.5);
 *   - a task is accepted only when the stage's free memory exceeds what the task needs (Section 4.4,
 *     Algorithm 1), and a task that allocates past its limit is stopped alone (memory limit, Section 4.5).
 * The paper's manager, worker and task are separate processes joined by RPC; here they are one worker thread
 * inside the calling process.
 *
 * Conventions
 *   - Every function returns an int: FR_OK (0) or a negative FR_ERR_* code; results come back through
 *     out-pointers.  No function throws, and a NULL required pointer gives FR_ERR_ARG.
 *   - "device pointer" means memory of the context's GPU; "host pointer" means ordinary process memory.
 *     The caller owns every buffer it passes in and keeps it alive until the object made from it is destroyed.
 *   - Streams are hipStream_t handles passed as void* (for example torch.cuda.Stream.cuda_stream); NULL is
 *     the default stream.
 *   - Times are uint64_t nanoseconds of CLOCK_MONOTONIC (fr_now_ns).
 *   - Task callbacks run on the library's worker thread only, never concurrently with each other.
 *   - One context serves one GPU and one stage; contexts are independent.  Calls on one context may come
 *     from any thread but fr_bubble_begin / fr_bubble_end must not race with each other.
 */
#ifndef FREERIDE_H
#define FREERIDE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------ status codes */
#define FR_OK            0
#define FR_ERR_ARG      (-1)   /* bad argument (NULL, out of range, shape the kernels do not support)       */
#define FR_ERR_STATE    (-2)   /* call not legal in the current state                                        */
#define FR_ERR_NOMEM    (-3)   /* task rejected at registration: not enough free memory (Algorithm 1)       */
#define FR_ERR_OOM      (-4)   /* task exceeded its memory limit and was stopped (Section 4.5)              */
#define FR_ERR_OVERRUN  (-5)   /* side work was still in flight when the bubble ended                        */
#define FR_ERR_HIP      (-6)   /* a HIP runtime call failed; fr_last_hip_error gives the code               */

/* Side-task states (Section 4.1). */
#define FR_SUBMITTED 0
#define FR_CREATED   1
#define FR_PAUSED    2
#define FR_RUNNING   3
#define FR_STOPPED   4

/* Event-log record kinds. */
#define FR_EV_INIT  1   /* the bubble was spent on InitSideTask                                             */
#define FR_EV_CHUNK 2   /* one step (a run of tiles) was enqueued in the bubble                             */
#define FR_EV_IDLE  3   /* the next step did not fit: rest of the bubble left idle ("insufficient time")    */
#define FR_EV_MISS  4   /* the step fitted the modelled budget but not the real clock; it was not launched  */
#define FR_EV_OVERRUN 5 /* fr_bubble_end found side work of the bubble still going on (written by that call) */
#define FR_EV_REFUSED 6 /* device gate: the tiles [tile0, tile1) of a step enqueued in the bubble were not done - the
                           whole step (too little time left when its kernel started, or a step behind such a one),
                           or the tail of a step that stopped between tiles, whose CHUNK record then ends at tile0;
                           the task was rewound to the first of them (one record per step)                          */

typedef struct fr_ctx fr_ctx;
typedef struct fr_alloc fr_alloc;
typedef int32_t fr_task_id;

/* ------------------------------------------------------------------ context */
typedef struct fr_config {
    int32_t  device_id;            /* HIP device ordinal.  -1 makes a host-only context: no HIP call is made,
                                      the side stream is NULL and fr_alloc_device takes memory from the host
                                      heap; meant for tasks that enqueue no GPU work (runtime tests).        */
    uint32_t cu_count;             /* side stream may use this many compute units (first cu_count mask bits,
                                      which the driver deals round-robin over the XCDs); 0 = use cu_mask.    */
    uint32_t cu_mask[8];           /* 256-bit CU mask for the side stream when cu_count == 0; all-zero, or a bit
                                      for every CU of the device = no mask (an ordinary stream on every CU). */
    uint64_t mem_available_bytes;  /* free device memory in this stage's bubbles (Section 2.2.1)             */
    uint64_t guard_ns;             /* modelled work must end this long before the declared bubble end        */
    uint64_t launch_cost_ns;       /* modelled fixed cost added to every step                                */
    uint64_t max_chunk_ns;         /* upper bound on one step's modelled cost; 0 = unbounded                 */
    uint32_t max_inflight;         /* steps enqueued but not yet finished on the GPU; 0 = default (8)        */
    uint32_t event_log_capacity;   /* records kept (oldest dropped first); 0 = default (65536)               */
    uint32_t time_steps;           /* N > 0: measure GPU time with HIP events around every group of N consecutive
                                      steps of a bubble (the last group of a bubble may be shorter); the group's time
                                      is reported on its last step's record.  1 times every step, at the price of
                                      about 3 us of GPU idle time between steps; 0 = no timing.                 */
    uint32_t adapt_costs;          /* nonzero: the profiler keeps running (Section 4.3): the timing groups of a bubble
                                      are summed and, before the next bubble is planned, update a cost scale for
                                      each of their cost classes (measured / modelled, taken at once when it
                                      rises, up to a doubling, and eased by 1/8 when it falls); a single group that
                                      took over 1.25 times its scaled cost also updates the scales at once, for the
                                      rest of its bubble (the update from the bubble's sums then starts from the
                                      scales before it).  Steps are planned against the scaled costs.  The plan then depends on
                                      measurements and no longer matches a plan computed ahead of time.  Needs
                                      time_steps.                                                              */
    uint32_t device_gate;          /* nonzero: every step also checks the GPU clock when its kernel starts and does
                                      nothing if it could not end gate_guard_ns before the bubble's declared end; a kernel
                                      that hands its tiles out checks again before every further tile and stops
                                      between tiles (freeride_device.h); what was not done is taken back
                                      (fr_task_ops.rewind) and logged as FR_EV_REFUSED.  Only for tasks that provide
                                      rewind.                                                                     */
    uint32_t gate_guard_ns;        /* the device gate's own guard: its deadline is the declared end minus this.  The
                                      host's guard_ns also has to cover steps that run slower than their model all
                                      bubble long; the gate reads the GPU's clock, so what is left for it to allow for
                                      is the error of one step's or tile's model and of the clock offset.  0 = guard_ns */
    uint64_t grace_ns;             /* framework-enforced limit (Section 4.5): a task whose work -- GPU steps, a step
                                      callback or InitSideTask -- is still going on this long after the end of the
                                      bubble it belongs to is stopped (FR_STOPPED, last_error FR_ERR_OVERRUN, memory
                                      released), as the paper's worker kills the task's process.  Checked at the next
                                      bubble notifications; 0 = never.                                           */
} fr_config;

int fr_create(const fr_config* cfg, fr_ctx** out);
/* Stops the task if any, joins the worker thread, destroys the side stream.  ctx is invalid afterwards. */
int fr_destroy(fr_ctx* ctx);
/* The side stream (hipStream_t) the library launches side-task work on; NULL for a host-only context. */
int fr_side_stream(fr_ctx* ctx, void** hip_stream_out);
/* Last failing HIP error code seen by this context (0 if none). */
int fr_last_hip_error(fr_ctx* ctx);
uint64_t fr_now_ns(void);

/* ------------------------------------------------------------------ side task */
typedef struct fr_step {
    uint64_t modelled_ns;   /* modelled cost of the step without launch_cost; 0 = nothing fits / no work    */
    uint64_t work_units;    /* task-defined amount of work in the step (PageRank: edges traversed)          */
    uint32_t run;           /* task-defined cursor of the step: restart count,                              */
    uint32_t segment;       /*   segment inside the run (a step never spans two segments),                  */
    uint32_t tile0, tile1;  /*   tile range [tile0, tile1) inside the segment                               */
    int32_t  finished;      /* plan_step sets 1 when the task has no work left at all                       */
    int32_t  completes_run; /* plan_step sets 1 when this step ends a run (PageRank: the K-th iteration)    */
    uint32_t cost_class;    /* 0..7: steps of one class share a cost scale when costs adapt (PageRank: the
                               segment kind)                                                                */
    /* filled in by the runtime before run_step when the device gate is on (gate == NULL otherwise): the
       arguments of fr_gate_admit for this step's kernels                                                    */
    uint32_t gate_slot;
    void*    gate;          /* device pointer to the context's fr_gate                                      */
    uint32_t gate_need_ticks;   /* the step's modelled duration in GPU wall-clock ticks                     */
    uint32_t gate_tile;     /* plan_step: modelled time, ns, a workgroup takes for the step's heaviest tile if the step's
                               kernel can stop between tiles (0 if it cannot: the step is all or nothing); the runtime
                               turns it into GPU wall-clock ticks, scaled like the step's cost, before run_step      */
} fr_step;

/*
 * The task's transition functions (Section 4.1).  `user` is the pointer given at registration.
 * create   : SUBMITTED -> CREATED, host-side set-up only.
 * init     : CREATED -> PAUSED, takes device memory through `a` (fr_alloc_device / fr_alloc_charge) and may
 *            enqueue set-up work on `stream`.  Runs inside the first bubble that finds the task CREATED.
 * plan_step: pure; describes the largest next step whose modelled cost + launch_cost_ns <= budget_ns.
 *            Sets modelled_ns = 0 when not even the smallest step fits.
 * run_step : RunNextStep(): enqueue exactly the planned step on `stream` and advance the cursor.
 * stop     : -> STOPPED, release everything taken in init (the accounting allocator frees what it handed out).
 * rewind   : optional (may be NULL).  Of the step `first_undone`, run_step of which has returned, only the first
 *            `tiles_done` tiles were done on the GPU (0: the device gate refused the step; more: its kernel
 *            stopped between tiles when the bubble's time ran out), and every step after it did nothing: the task's
 *            cursor goes back to the first tile not done, and *work_units_done_out receives the work units of
 *            the tiles that were.
 * Each returns FR_OK or an FR_ERR_* code; a failure stops the task.
 */
typedef struct fr_task_ops {
    int (*create)(void* user);
    int (*init)(void* user, fr_alloc* a, void* stream);
    int (*plan_step)(void* user, uint64_t budget_ns, uint64_t launch_cost_ns, fr_step* out);
    int (*run_step)(void* user, void* stream, const fr_step* planned);
    int (*stop)(void* user);
    int (*rewind)(void* user, const fr_step* first_undone, uint32_t tiles_done, uint64_t* work_units_done_out);
} fr_task_ops;

/* The side-task profile (Section 4.3): memory need and shortest step. */
typedef struct fr_task_profile {
    uint64_t mem_limit_bytes;   /* what the task may allocate; also what Algorithm 1 compares            */
    uint64_t min_step_ns;       /* modelled cost of the task's smallest step (informational)             */
} fr_task_profile;

/*
 * Algorithm 1 for one worker: the task is accepted only if ctx.mem_available_bytes > profile.mem_limit_bytes
 * (strictly); otherwise FR_ERR_NOMEM.  An accepted task joins the worker's queue (SUBMITTED).  Algorithm 2: when
 * the worker has no live current task the head of the queue becomes current, create() runs (on the thread that
 * makes it current: the caller of this function or of fr_task_stop, or the worker thread) and the task is
 * CREATED; if create() fails the task is dropped (from this call: its error is returned).  The current task
 * gives way to the next one when it stops, or when its plan_step reports `finished` while others are waiting.
 * `ops` is copied.  fr_query_progress works for every id this context has handed out.
 */
int fr_task_register(fr_ctx* ctx, const fr_task_ops* ops, void* user, const fr_task_profile* profile,
                     fr_task_id* id_out);
/* StopSideTask(): legal from CREATED, PAUSED and RUNNING; waits for side work in flight, then calls stop().
   A task still waiting in the queue (SUBMITTED) just leaves it.  FR_ERR_STATE if already stopped. */
int fr_task_stop(fr_ctx* ctx, fr_task_id id);

/*
 * Accounting allocator handed to init().  fr_alloc_device returns device memory (256-byte aligned) or NULL;
 * once the running total would pass the task's mem_limit_bytes it returns NULL and latches an out-of-memory
 * condition, after which the runtime stops the task with FR_ERR_OOM and the stage is untouched.
 * fr_alloc_charge only books `bytes` against the limit (for buffers the caller handed to the task); it
 * returns FR_OK or FR_ERR_OOM.  Memory handed out is freed by the runtime after stop().
 */
void* fr_alloc_device(fr_alloc* a, size_t bytes);
int   fr_alloc_charge(fr_alloc* a, size_t bytes);
/* Returns a block taken with fr_alloc_device before the task stops (set-up scratch); FR_ERR_ARG if unknown. */
int   fr_alloc_free(fr_alloc* a, void* p);
uint64_t fr_alloc_used(const fr_alloc* a);
uint64_t fr_alloc_peak(const fr_alloc* a);   /* highest value fr_alloc_used has reached */

/*
 * Bubble notifications from the stage's scheduler (Section 3.2: start timestamp and duration).
 * fr_bubble_begin: a bubble of declared length `duration_ns` opened at `t_begin_ns`.  If the task is CREATED
 *   it is initialised in this bubble; if PAUSED it is started and steps are planned against
 *   duration_ns - guard_ns.  FR_ERR_STATE if a bubble is already open.
 * fr_bubble_end: PauseSideTask().  Returns once the worker has stopped enqueuing.  FR_ERR_OVERRUN (also
 *   counted) if side work is still in flight on the GPU (and stays so for 20 us), or if InitSideTask or a step callback is
 *   still running (the call does not wait for InitSideTask at all and for a step callback only 0.2 ms past the
 *   bubble's declared end; bubbles that open before it returns are seen but not used).  With grace_ns set, work
 *   that is still going on grace_ns later gets the task stopped.  FR_ERR_STATE if no bubble is open.
 */
int fr_bubble_begin(fr_ctx* ctx, uint64_t t_begin_ns, uint64_t duration_ns);
int fr_bubble_end(fr_ctx* ctx);

typedef struct fr_progress {
    int32_t  state;                 /* FR_SUBMITTED .. FR_STOPPED                                          */
    int32_t  last_error;            /* FR_OK or the error that stopped the task                            */
    uint64_t runs_completed;
    uint64_t work_units_done;       /* summed over enqueued steps                                          */
    uint64_t steps;                 /* steps enqueued                                                      */
    uint64_t bubbles_seen;
    uint64_t bubbles_used;          /* bubbles in which at least one step ran                              */
    uint64_t ns_bubble_declared;    /* sum of declared bubble lengths                                      */
    uint64_t ns_modelled;           /* sum of modelled step costs, launch_cost included                    */
    uint64_t ns_measured;           /* sum of measured GPU time of steps (time_steps != 0), resolved so far */
    uint64_t ns_idle_insufficient;  /* modelled time left idle because the next step did not fit           */
    uint64_t overruns;
    uint64_t deadline_misses;
    uint64_t mem_used_bytes;
    uint64_t killed;                /* 1 if the framework-enforced limit stopped the task                  */
    uint64_t steps_refused;         /* steps the device gate refused or cut short; what they did not do leaves
                                       steps / work_units_done / runs_completed again once the bubble's GPU
                                       work has drained                                                    */
} fr_progress;
int fr_query_progress(fr_ctx* ctx, fr_task_id id, fr_progress* out);

typedef struct fr_event {
    uint32_t kind;          /* FR_EV_*                                                                      */
    uint32_t bubble;        /* 0-based index of the bubble since fr_create                                  */
    uint32_t run, segment, tile0, tile1;
    uint64_t modelled_ns;   /* CHUNK/MISS: step cost + launch_cost; IDLE: modelled time left; INIT: 0       */
    uint64_t work_units;
    uint64_t t_host_ns;     /* host clock when the record was made                                          */
    uint64_t measured_ns;   /* CHUNK, last step of a timing group (every step if time_steps == 1): GPU time of the
                               group, from the previous group's end (or the bubble's first launch) to this step's
                               end; 0 on the group's other steps, if not timed, or if not finished yet      */
} fr_event;
/* Copies up to `cap` of the oldest retained records in order; *n_out = number copied.  Resolves finished
   step timings first.  Does not consume the log; fr_event_log_clear does. */
int fr_event_log(fr_ctx* ctx, fr_event* buf, size_t cap, size_t* n_out);
int fr_event_log_clear(fr_ctx* ctx);

/*
 * The program-directed fit rule as a pure function (Section 4.5): given the cumulative costs
 * prefix[0..n] (prefix[0] = 0, prefix[i] = cost of tiles 0..i-1) of one segment, the first tile `tile0`
 * still to do and a budget, returns through *n_fit the largest n with
 * launch_cost_ns + prefix[tile0 + n] - prefix[tile0] <= budget_ns (0 when not even one tile fits).
 */
int fr_chunk_fit(const uint64_t* prefix, uint32_t n_tiles, uint32_t tile0, uint64_t budget_ns,
                 uint64_t launch_cost_ns, uint32_t* n_fit);

/*
 * Cost adaptation (fr_config.adapt_costs).  Scales are parts per million of the current task's own modelled cost,
 * 1000000 when a task becomes the worker's current one, kept within [250000, 16000000].
 * fr_cost_scale_next: the update rule as a pure function: with r = measured_ns / modelled_ns (in ppm, clamped to
 *   the range above; the old scale if modelled_ns is 0) the new scale is min(r, 2 * scale_ppm) if
 *   r >= scale_ppm, else scale_ppm - (scale_ppm - r) / 8.
 * fr_cost_scales: the context's eight current scales (host array of 8).
 */
uint32_t fr_cost_scale_next(uint32_t scale_ppm, uint64_t modelled_ns, uint64_t measured_ns);
int fr_cost_scales(fr_ctx* ctx, uint32_t* scales_ppm_out);

/* ------------------------------------------------------------------ the PageRank side task */
/*
 * Pull-based PageRank over an in-edge CSR, fp32 ranks, fixed iteration count, dangling mass spread uniformly,
 * Jacobi iterations (the paper's graph-analytics side task, Section 6.1.4; one iteration = one pass over the
 * graph, Section 6.2).  InitSideTask rebuilds the CSR into a partition-centric layout on the GPU (vertices
 * renumbered by in-degree, rows cut into ranges); work is cut into tiles fixed at that point and results do not
 * depend on how tiles are grouped into launches.  A launch has at most as many workgroups as the stream's compute
 * units run side by side; if it holds more tiles, its workgroups hand them out among themselves.  The layout is cut
 * for the compute units of the stream InitSideTask runs on, and the last bit of a rank may differ between layouts.
 * A run is the segment sequence  V0, S_0, G_0, S_1, G_1, ..., S_{K-1}, G_{K-1}, F  where
 *   V0  (vertex pass)  r_0 = 1/V: per-tile partial sums of dangling r_0;
 *   S_k (scatter)      one message contrib_k[u] = r_k[u] / outdeg[u] per (range, source u) pair; for k > 0 it first
 *                      finishes the rows that no gather tile could finish alone (ranges cut into several gather
 *                      tiles, and ranges without in-edges);
 *   G_k (gather)       acc_k[v] = sum over v's in-edges of the source's message, then for the rows of a range with
 *                      one gather tile r_{k+1} = base_k + d * acc_k, contrib_{k+1}, dangling partials;
 *                      base_k = (1 - d)/V + d * D_k / V, D_k = sum of the dangling partials of r_k;
 *   F   (finish)       r_K of the rows S would have finished, once, after the last iteration.
 * The last iteration writes r_K to ranks_out.  With K = 0 the run is V0 alone, which writes r_0 there.
 */
#define FR_PR_SEG_VERTEX  0
#define FR_PR_SEG_SCATTER 1
#define FR_PR_SEG_GATHER  2
#define FR_PR_SEG_FINISH  3

typedef struct fr_pagerank_desc {
    int64_t  n_vertices;          /* V >= 1                                                                 */
    int64_t  n_edges;             /* E >= 0, below 2^31                                                     */
    const int32_t* row_ptr;       /* device, V + 1 entries: in-edge CSR row starts                          */
    const int32_t* col;           /* device, E entries: source of each in-edge                              */
    const int32_t* out_degree;    /* device, V entries: edges leaving each vertex, with multiplicity        */
    float*   ranks_out;           /* device, V entries: r_K of the latest completed run                     */
    float    damping;
    int32_t  iterations;          /* K >= 0                                                                 */
    int32_t  max_runs;            /* stop harvesting after this many completed runs; 0 = restart forever    */
    int32_t  reserved;
    uint64_t mem_limit_bytes;     /* the task's memory limit; caller buffers above are booked against it    */
    /* cost model, integer femtoseconds (a streaming kernel spends about 1000 fs on an edge, so picoseconds would
       be too coarse), fixed for the task's life (0 = library default); tile cost in ns = ceil(sum / 10^6), at least 1:
         vertex tile  : rows * fs_per_vertex
         scatter tile : (messages + values read for its sources) * fs_per_message, where a source costs one
                        value (its contribution or 1/outdeg) and, in a range cut into several gather
                        pieces, one partial sum per piece more (the weight the tiles are cut by)
         gather tile  : weight * fs_per_edge / 2, weight = 2 * edges + 6 * repeated edges + 147456 per piece
                        (a piece is a run of edges of one range: a heavy range is cut into several, each a tile of
                        its own; light ones share a tile.  A repeated edge has the same source and row as the edge
                        before it: the two collide in the accumulator.  The constant stands for the start and the
                        row pass of a piece.)
         finish tile  : finish_tile_ns (already ns)                                                         */
    uint64_t fs_per_edge;
    uint64_t fs_per_message;
    uint64_t fs_per_vertex;
    uint64_t finish_tile_ns;
    /* Shortest step per segment kind (indexed by FR_PR_SEG_*), ns; 0 = none.  A launch of a few tiles takes about
       as long as one tile alone (the tiles run side by side), so the modelled cost of a step is
       max(sum of its tile costs, min_step_ns[kind]), and a step is only planned if that fits.  A sweep's tiles run
       `slots` at a time (fr_pagerank_info_t): a step of more tiles than that which does not reach the segment's end
       is a whole number of rounds, and a step of n <= slots tiles, which fills only part of the slots, is modelled as
       max(min_step_ns[kind], sum of its tile costs + min_step_ns[kind] * (full - n) / full), full = min(slots,
       tiles of the sweep) - between one tile alone (the floor) and a full round (the sum) the time was measured to
       grow linearly with n - with n taken down until that fits.                                                  */
    uint64_t min_step_ns[4];
    /* Partition sizes of the layout: destination rows per range (8192 or 16384) and the most source vertices of a
       scatter tile (16384 or 32768); 0 = chosen by the library (16384 rows from 2^22 vertices on, 32768 sources
       from 2^24 vertices on).  Other values: FR_ERR_ARG at InitSideTask.                                                */
    uint32_t rows_per_partition;
    uint32_t sources_per_partition;
} fr_pagerank_desc;

/* Facts about the layout built by InitSideTask. */
typedef struct fr_pagerank_info_t {
    uint64_t messages;            /* distinct (range, source) pairs                                         */
    uint32_t ranges;              /* row ranges, ceil(V / rows_per_partition)                               */
    uint32_t scatter_tiles;       /* one source interval (a piece), or several light ones on small graphs   */
    uint32_t gather_tiles;        /* one piece (a run of edges of one range), or several light ones on small graphs */
    uint32_t merged_ranges;       /* ranges cut into several gather pieces                                  */
    uint32_t nonempty_ranges;     /* ranges with in-edges (they come first: rows are ordered by in-degree)  */
    uint32_t rows_per_partition;  /* destination rows per range                                             */
    uint32_t sources_per_partition; /* most source vertices of a scatter tile                               */
    uint32_t partial_rows;        /* gather pieces of merged ranges (rows of fp32 partial sums)             */
    uint64_t bytes_resident;      /* booked against the limit after init (caller buffers included)          */
    uint64_t bytes_peak;          /* highest amount booked during init (set-up scratch included)            */
    uint32_t scatter_slots;       /* workgroups of a scatter launch / of a gather launch that run side by side on  */
    uint32_t gather_slots;        /* the stream's compute units: a step of more tiles runs in rounds, and plan_step
                                     cuts a step that does not reach its segment's end to whole rounds             */
} fr_pagerank_info_t;

/* Builds the task object and fills in the callbacks and profile to register with.  No device work yet. */
int fr_pagerank_make(const fr_pagerank_desc* d, fr_task_ops* ops_out, void** user_out, fr_task_profile* prof_out);
/* Frees the task object; only after fr_task_stop (or if it was never registered). */
int fr_pagerank_destroy(void* user);
/* The four calls below need the layout, so they return FR_ERR_STATE until InitSideTask has run. */
int fr_pagerank_info(void* user, fr_pagerank_info_t* out);
/* Number of tiles of a segment kind (FR_PR_SEG_*), their modelled costs in ns, and the work they hold
   (vertex: rows, scatter: messages, gather: edges, finish: 0). */
int fr_pagerank_tiles(void* user, int32_t seg_kind, uint32_t* n_tiles_out);
int fr_pagerank_tile_costs(void* user, int32_t seg_kind, uint32_t* costs_host, size_t cap, size_t* n_out);
int fr_pagerank_tile_work(void* user, int32_t seg_kind, uint64_t* work_host, size_t cap, size_t* n_out);
/* The tiles' multiplicands in the cost formulas above: gather: the weight; scatter: values read for the sources
   (messages not included: those are the tile's work); vertex: rows; finish: 0. */
int fr_pagerank_tile_weights(void* user, int32_t seg_kind, uint64_t* weights_host, size_t cap, size_t* n_out);
/*
 * Runs one whole run (K iterations) outside any bubble on `stream`, at most `max_tiles_per_launch` tiles per
 * kernel launch (0 = a whole segment per launch), waits for it and leaves r_K in ranks_out.  Same kernels and
 * tiles as the harvested path: the reference for the "any chunking gives the same bits" property.  The task
 * must not be registered with a context (it initialises itself against its own mem_limit_bytes on `device_id`).
 * phase_ns_out (host, 4 entries indexed by FR_PR_SEG_*, may be NULL) receives the summed GPU time per segment kind.
 */
int fr_pagerank_run_standalone(void* user, int32_t device_id, void* stream, uint32_t max_tiles_per_launch,
                               uint64_t* phase_ns_out);
/*
 * For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid it): the same run as fr_pagerank_run_standalone with the same kernels and tiles, hence the same bits in
 * ranks_out, but the run's working memory (messages, contributions, dangling partials, partial sums) lies in a
 * 64 MiB array inside the library's device code, of which every GPU holds its own copy until the process ends.  Makes no
 * hipMalloc / hipFree and creates no events; it does wait for the stream.  The task's layout must have been built
 * before by fr_pagerank_run_standalone on the same device (FR_ERR_STATE otherwise; this call builds nothing), and the
 * task must not be registered with a context.  FR_ERR_ARG if the working memory of this graph does not fit the array
 * (it needs about 4 bytes per message and per vertex plus 65536 per partial-sum row, each part rounded up to 256), or if device_id is not in 0 .. 63.
 * All calls on one GPU share the array, which keeps the last call's contents (every part is written before it is
 * read, so nothing needs clearing): calls that overlap in time on one GPU race; run them one after the other.
 */
int fr_pagerank_run_standalone_noalloc(void* user, int32_t device_id, void* stream, uint32_t max_tiles_per_launch);

/* ------------------------------------------------------------------ Graph SGD side task */
/*
 * Stochastic gradient descent for matrix factorization over a rating graph: the second graph workload of
 * Section 6.1.4 (one iteration = one pass over the graph, Section 6.2).  The paper names the method only; the
 * arithmetic is the textbook one (Koren, Bell, Volinsky 2009), for every rating r_ui, one after the other,
 *     e = r_ui - <p_u, q_i>,   p_u += gamma (e q_i - lambda p_u),   q_i += gamma (e p_u - lambda q_i),
 * and the order is stratified (Gemulla et al. 2011): users and items in `blocks` blocks of consecutive ids holding
 * about E / blocks ratings each (block k begins at the first id with ceil(k E / blocks) or more ratings before it;
 * a block may be empty); cell (a, b) = ratings of user block a and item block b; an iteration = `blocks` strata, stratum
 * s = cells (a, (a + s) mod blocks), which share no factor row and run side by side; inside a cell by user, then
 * by item.  All roundings of an update are fixed: t_l = p_l * q_l; in rounds w = 1, 2, 4, .. t_l += t_(l xor w);
 * e = r - t; ge = gamma * e; gl = gamma * lambda; p_l' = fma(ge, q_l, fma(-gl, p_l, p_l)); q_l' likewise from the
 * old p_l - so the factors are the same bits however the cells are grouped into steps.
 *
 * As a side task: one run = `iterations` iterations = iterations * blocks segments (a segment is a stratum, a
 * tile is a cell); the factors carry over from run to run.  work_units = ratings visited.
 * Modelled cost of a cell = ceil(ratings * fs_per_rating / 10^6) ns, at least 1; of a step =
 * max(sum over its cells, min_step_ns, ceil(ratings of its largest cell * fs_per_chain_rating / 10^6)): the cells of
 * a step run side by side, each a chain of dependent updates, so a step takes as long as its largest cell, and
 * strata differ in that by a factor of two and more.  A step is the largest run of cells whose sum fits; if the
 * chain term then does not fit, nothing is planned.
 */
typedef struct fr_sgd_desc {
    int64_t  n_users;             /* U >= 1, below 2^27 - 1024                                              */
    int64_t  n_items;             /* I >= 1, below 2^27 - 1024                                              */
    int64_t  n_ratings;           /* E >= 0, below 2^31                                                     */
    const int32_t* row_ptr;       /* device, U + 1 entries: ratings as CSR by user                          */
    const int32_t* item;          /* device, E entries: ascending and distinct inside a row (FR_ERR_ARG from
                                     InitSideTask otherwise); only read                                     */
    const float*   rating;        /* device, E entries; only read                                           */
    float*   P;                   /* device, U x factors, row-major: in and out                             */
    float*   Q;                   /* device, I x factors, row-major: in and out                             */
    int32_t  factors;             /* F: 16, 32 or 64                                                        */
    int32_t  blocks;              /* B: 1 .. 1024; 0 = chosen by the library (cells of 32 ratings or more)   */
    float    gamma;               /* step length, >= 0                                                      */
    float    lambda;              /* regularisation, >= 0                                                   */
    int32_t  iterations;          /* K >= 1 iterations per run                                              */
    int32_t  max_runs;            /* stop harvesting after this many runs; 0 = keep training forever        */
    uint64_t mem_limit_bytes;     /* the task's memory limit; caller buffers above are booked against it    */
    uint64_t fs_per_rating;       /* cost model, femtoseconds (0 = library default)                         */
    uint64_t min_step_ns;         /* shortest step, ns (0 = none)                                           */
    uint64_t fs_per_chain_rating; /* femtoseconds per rating of a step's largest cell (0 = term not used)   */
} fr_sgd_desc;

typedef struct fr_sgd_info_t {
    uint32_t blocks;              /* B in use                                                               */
    uint32_t reserved[2];
    uint32_t largest_cell;        /* ratings in the largest cell                                            */
    uint64_t chain_ratings;       /* sum over the strata of their largest cell: the critical path of one
                                     iteration, in ratings                                                  */
    uint64_t bytes_resident;      /* booked after InitSideTask, caller buffers included                     */
    uint64_t bytes_peak;          /* highest booking during InitSideTask                                    */
} fr_sgd_info_t;

/* Fills ops / profile for fr_task_register; *user_out is the task object (host).  Nothing touches the GPU yet. */
int fr_sgd_make(const fr_sgd_desc* d, fr_task_ops* ops_out, void** user_out, fr_task_profile* prof_out);
/* Frees the task object; FR_ERR_STATE while it is registered with a context (stop it first). */
int fr_sgd_destroy(void* user);
/* The two calls below need the layout: FR_ERR_STATE until InitSideTask has run. */
int fr_sgd_info(void* user, fr_sgd_info_t* out);
/* First ids of the user blocks (items = 0) or item blocks (items = 1): B + 1 entries; *n_out = B + 1. */
int fr_sgd_block_starts(void* user, int32_t items, uint32_t* starts_host, size_t cap, size_t* n_out);
/* Ratings in the cells (a, (a + stratum) mod B), a = 0 .. B - 1; *n_out = B. */
int fr_sgd_cell_sizes(void* user, uint32_t stratum, uint32_t* sizes_host, size_t cap, size_t* n_out);
/*
 * Runs one whole run (K iterations) outside any bubble on `stream`, at most `max_cells_per_launch` cells per
 * kernel launch (0 = a whole stratum per launch), and waits for it.  Same kernel and cells as the harvested
 * path.  The task must not be registered with a context.  ns_out (host, may be NULL) receives the GPU time.
 */
int fr_sgd_run_standalone(void* user, int32_t device_id, void* stream, uint32_t max_cells_per_launch, uint64_t* ns_out);

/* ------------------------------------------------------------------ stage load and stage emulator */
#define FR_LOAD_BUSYWAIT 0   /* one small kernel that spins on the GPU clock for fp_ns / bp_ns              */
#define FR_LOAD_GPT      1   /* bf16 MFMA GEMM bursts shaped like `layers` transformer blocks               */

typedef struct fr_load fr_load;
typedef struct fr_load_desc {
    int32_t  kind;
    int32_t  layers, hidden, ffn, tokens;   /* FR_LOAD_GPT: all multiples of 256                            */
    uint64_t fp_ns, bp_ns;                  /* FR_LOAD_BUSYWAIT                                             */
    void*    workspace;                     /* device; FR_LOAD_GPT operands live here (bf16)                */
    uint64_t workspace_bytes;
    uint64_t seed;
} fr_load_desc;
int fr_load_workspace_bytes(const fr_load_desc* d, uint64_t* bytes_out);
/* FR_LOAD_GPT fills the workspace with seeded values on `stream` (may be NULL) and waits for it. */
int fr_load_make(const fr_load_desc* d, void* stream, fr_load** out);
int fr_load_destroy(fr_load* l);
/* Enqueue one forward / backward burst on `stream`: FP = 4 GEMMs per layer (QKV, projection, FFN up, FFN
   down), BP = the 8 matching data- and weight-gradient GEMMs per layer. */
int fr_load_fp(fr_load* l, void* stream);
int fr_load_bp(fr_load* l, void* stream);
/* Part `part` of `parts` of a burst (kind 0 = FP, 1 = BP): the GEMMs of the layers [part * layers / parts,
   (part + 1) * layers / parts) (parts must divide layers), or a busy-wait of 1 / parts of the burst's time: what
   one model chunk of an interleaved schedule runs.  parts = 1 is the whole burst. */
int fr_load_part(fr_load* l, void* stream, int32_t kind, int32_t part, int32_t parts);
/* Floating-point operations of one FP / BP burst (2 M N K per GEMM); 0 for busy-wait loads. */
int fr_load_flops(fr_load* l, uint64_t* fp_flops_out, uint64_t* bp_flops_out);

/*
 * C[M, N] (bf16, row-major) = A[M, K] (bf16, row-major) x B[N, K]^T (bf16, row-major, i.e. both operands
 * K-contiguous), fp32 accumulation on the MFMA units.  M, N multiples of 256 and K a multiple of 64, else
 * FR_ERR_ARG.  All pointers device, 16-byte aligned.  Asynchronous on `stream`.
 */
int fr_gemm_bf16(const void* A, const void* B, void* C, int32_t M, int32_t N, int32_t K, void* stream);

#define FR_SCHED_1F1B  0
#define FR_SCHED_GPIPE 1
#define FR_SCHED_INTERLEAVED 2   /* interleaved 1F1B (Narayanan et al. 2021), one of the bubble-reducing schedules
                                    Sections 1 and 2.2.2 name: the stage holds `chunks` model chunks, an operation is
                                    one chunk's FP or BP; the bubbles add up to 1 / chunks of the plain schedule's,
                                    in more and shorter windows.  m must be a multiple of p.                         */
typedef struct fr_stage fr_stage;
typedef struct fr_stage_desc {
    int32_t  schedule;      /* FR_SCHED_*                                                                   */
    int32_t  p, m, stage;   /* pipeline depth, micro-batches per epoch, emulated stage (0-based)            */
    uint64_t f_ns, b_ns;    /* declared FP / BP durations of one operation on every stage (FR_SCHED_INTERLEAVED: of
                               one chunk): fix the waits that stand for the other stages and the declared
                               bubble lengths                                                               */
    int32_t  chunks;        /* FR_SCHED_INTERLEAVED: model chunks per stage, 1 .. 64, a divisor of the load's
                               layers; otherwise 0 or 1                                                     */
    int32_t  reserved;
} fr_stage_desc;
typedef struct fr_stage_op {
    int32_t  kind;          /* 0 = FP, 1 = BP                                                               */
    int32_t  microbatch;
    uint64_t start_ns, end_ns;      /* in the ideal schedule, from the epoch start                          */
    uint64_t bubble_before_ns;      /* idle time in front of this operation (0 = none)                      */
    int32_t  chunk;                 /* model chunk (FR_SCHED_INTERLEAVED), else 0                           */
    int32_t  reserved;
} fr_stage_op;
typedef struct fr_epoch_result {
    uint64_t epoch_ns;          /* wall time of the epoch on this stage                                      */
    uint64_t busy_ns;           /* sum of measured FP/BP burst times                                         */
    uint64_t bubble_ns;         /* sum of declared bubble lengths                                            */
    uint32_t n_ops, n_bubbles;
    uint32_t overruns;          /* fr_bubble_end calls that reported FR_ERR_OVERRUN                          */
    uint32_t reserved;
} fr_epoch_result;
/* Emulates one stage of a pipeline (Section 2.1): its operation order with the waits the other stages would
   impose.  `load` supplies the FP/BP work; `stage_stream` is the stream it runs on. */
int fr_stage_make(const fr_stage_desc* d, fr_load* load, void* stage_stream, fr_stage** out);
int fr_stage_destroy(fr_stage* s);
/* The stage's operations in order with ideal start/end times; *epoch_ns_out = ideal epoch length;
   *tail_bubble_ns_out = idle time after the last operation. */
int fr_stage_ops(fr_stage* s, fr_stage_op* buf, size_t cap, size_t* n_out, uint64_t* epoch_ns_out,
                 uint64_t* tail_bubble_ns_out);
/* Runs one epoch: each operation's burst is enqueued and waited for; each bubble is reported to `ctx`
   (may be NULL: nothing is reported, the stage just waits) with fr_bubble_begin, waited out on the host
   clock, and closed with fr_bubble_end. */
int fr_stage_run_epoch(fr_stage* s, fr_ctx* ctx, fr_epoch_result* out);
/*
 * For measuring the stage's slowdown (Section 6.1.5: I = (T_with - T_no) / T_no).  A GPU whose bubbles are idle
 * may run its next burst at other clocks than one whose bubbles are harvested, which an A/B of "with side task"
 * against "idle bubbles" cannot tell from interference.  With a filler set, epochs run with ctx == NULL fill every
 * bubble longer than guard_ns with a kernel of `workgroups` workgroups of 256 threads on `stream` that does
 * register-only arithmetic for the bubble's length minus guard_ns (no memory traffic; it ends by the GPU clock, or
 * by a trip cap), and wait for it at the bubble's end: a baseline that differs from a harvested epoch by the side
 * task's memory traffic only.  workgroups = 0 switches the filler off.  Epochs with a ctx are not affected.
 */
int fr_stage_set_filler(fr_stage* s, void* stream, uint32_t workgroups, uint64_t guard_ns);
/* Host-clock durations (enqueue to completion) of the latest epoch's operations, in the order of fr_stage_ops;
   *n_out = their number. */
int fr_stage_op_times(fr_stage* s, uint64_t* ns_host, size_t cap, size_t* n_out);

#ifdef __cplusplus
}
#endif
#endif /* FREERIDE_H */
