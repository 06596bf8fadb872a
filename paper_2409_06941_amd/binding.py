"""ctypes declarations mirroring include/freeride.h, plus small object wrappers that only marshal arguments."""
import ctypes as C
import os

from . import build as _build

LIB_PATH = _build.LIB

FR_OK, FR_ERR_ARG, FR_ERR_STATE, FR_ERR_NOMEM, FR_ERR_OOM, FR_ERR_OVERRUN, FR_ERR_HIP = 0, -1, -2, -3, -4, -5, -6
FR_SUBMITTED, FR_CREATED, FR_PAUSED, FR_RUNNING, FR_STOPPED = range(5)
FR_EV_INIT, FR_EV_CHUNK, FR_EV_IDLE, FR_EV_MISS, FR_EV_OVERRUN, FR_EV_REFUSED = 1, 2, 3, 4, 5, 6
FR_PR_SEG_VERTEX, FR_PR_SEG_SCATTER, FR_PR_SEG_GATHER, FR_PR_SEG_FINISH = 0, 1, 2, 3
FR_LOAD_BUSYWAIT, FR_LOAD_GPT = 0, 1
FR_SCHED_1F1B, FR_SCHED_GPIPE, FR_SCHED_INTERLEAVED = 0, 1, 2

_ERR_NAMES = {0: "FR_OK", -1: "FR_ERR_ARG", -2: "FR_ERR_STATE", -3: "FR_ERR_NOMEM", -4: "FR_ERR_OOM",
              -5: "FR_ERR_OVERRUN", -6: "FR_ERR_HIP"}


class FreeRideError(RuntimeError):
    def __init__(self, code, where):
        super().__init__("%s returned %s" % (where, _ERR_NAMES.get(code, code)))
        self.code = code


class fr_config(C.Structure):
    _fields_ = [("device_id", C.c_int32), ("cu_count", C.c_uint32), ("cu_mask", C.c_uint32 * 8),
                ("mem_available_bytes", C.c_uint64), ("guard_ns", C.c_uint64), ("launch_cost_ns", C.c_uint64),
                ("max_chunk_ns", C.c_uint64), ("max_inflight", C.c_uint32), ("event_log_capacity", C.c_uint32),
                ("time_steps", C.c_uint32), ("adapt_costs", C.c_uint32), ("device_gate", C.c_uint32), ("gate_guard_ns", C.c_uint32),
                ("grace_ns", C.c_uint64)]


class fr_step(C.Structure):
    _fields_ = [("modelled_ns", C.c_uint64), ("work_units", C.c_uint64), ("run", C.c_uint32), ("segment", C.c_uint32),
                ("tile0", C.c_uint32), ("tile1", C.c_uint32), ("finished", C.c_int32), ("completes_run", C.c_int32),
                ("cost_class", C.c_uint32), ("gate_slot", C.c_uint32), ("gate", C.c_void_p), ("gate_need_ticks", C.c_uint32),
                ("gate_tile", C.c_uint32)]


CREATE_FN = C.CFUNCTYPE(C.c_int, C.c_void_p)
INIT_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_void_p, C.c_void_p)
PLAN_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_uint64, C.c_uint64, C.POINTER(fr_step))
RUN_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_void_p, C.POINTER(fr_step))
STOP_FN = C.CFUNCTYPE(C.c_int, C.c_void_p)
REWIND_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.POINTER(fr_step), C.c_uint32, C.POINTER(C.c_uint64))


class fr_task_ops(C.Structure):
    _fields_ = [("create", CREATE_FN), ("init", INIT_FN), ("plan_step", PLAN_FN), ("run_step", RUN_FN), ("stop", STOP_FN),
                ("rewind", REWIND_FN)]


class fr_task_profile(C.Structure):
    _fields_ = [("mem_limit_bytes", C.c_uint64), ("min_step_ns", C.c_uint64)]


class fr_progress(C.Structure):
    _fields_ = [("state", C.c_int32), ("last_error", C.c_int32), ("runs_completed", C.c_uint64),
                ("work_units_done", C.c_uint64), ("steps", C.c_uint64), ("bubbles_seen", C.c_uint64),
                ("bubbles_used", C.c_uint64), ("ns_bubble_declared", C.c_uint64), ("ns_modelled", C.c_uint64),
                ("ns_measured", C.c_uint64), ("ns_idle_insufficient", C.c_uint64), ("overruns", C.c_uint64),
                ("deadline_misses", C.c_uint64), ("mem_used_bytes", C.c_uint64), ("killed", C.c_uint64),
                ("steps_refused", C.c_uint64)]


class fr_event(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("bubble", C.c_uint32), ("run", C.c_uint32), ("segment", C.c_uint32),
                ("tile0", C.c_uint32), ("tile1", C.c_uint32), ("modelled_ns", C.c_uint64), ("work_units", C.c_uint64),
                ("t_host_ns", C.c_uint64), ("measured_ns", C.c_uint64)]


class fr_pagerank_desc(C.Structure):
    _fields_ = [("n_vertices", C.c_int64), ("n_edges", C.c_int64), ("row_ptr", C.c_void_p), ("col", C.c_void_p),
                ("out_degree", C.c_void_p), ("ranks_out", C.c_void_p), ("damping", C.c_float), ("iterations", C.c_int32),
                ("max_runs", C.c_int32), ("reserved", C.c_int32), ("mem_limit_bytes", C.c_uint64),
                ("fs_per_edge", C.c_uint64), ("fs_per_message", C.c_uint64), ("fs_per_vertex", C.c_uint64),
                ("finish_tile_ns", C.c_uint64), ("min_step_ns", C.c_uint64 * 4),
                ("rows_per_partition", C.c_uint32), ("sources_per_partition", C.c_uint32)]


class fr_pagerank_info_t(C.Structure):
    _fields_ = [("messages", C.c_uint64), ("ranges", C.c_uint32), ("scatter_tiles", C.c_uint32),
                ("gather_tiles", C.c_uint32), ("merged_ranges", C.c_uint32), ("nonempty_ranges", C.c_uint32),
                ("rows_per_partition", C.c_uint32), ("sources_per_partition", C.c_uint32), ("partial_rows", C.c_uint32),
                ("bytes_resident", C.c_uint64), ("bytes_peak", C.c_uint64), ("scatter_slots", C.c_uint32),
                ("gather_slots", C.c_uint32)]


class fr_sgd_desc(C.Structure):
    _fields_ = [("n_users", C.c_int64), ("n_items", C.c_int64), ("n_ratings", C.c_int64), ("row_ptr", C.c_void_p),
                ("item", C.c_void_p), ("rating", C.c_void_p), ("P", C.c_void_p), ("Q", C.c_void_p),
                ("factors", C.c_int32), ("blocks", C.c_int32), ("gamma", C.c_float), ("lam", C.c_float),
                ("iterations", C.c_int32), ("max_runs", C.c_int32), ("mem_limit_bytes", C.c_uint64),
                ("fs_per_rating", C.c_uint64), ("min_step_ns", C.c_uint64), ("fs_per_chain_rating", C.c_uint64)]


class fr_sgd_info_t(C.Structure):
    _fields_ = [("blocks", C.c_uint32), ("reserved", C.c_uint32 * 2),
                ("largest_cell", C.c_uint32), ("chain_ratings", C.c_uint64), ("bytes_resident", C.c_uint64),
                ("bytes_peak", C.c_uint64)]


class fr_load_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("layers", C.c_int32), ("hidden", C.c_int32), ("ffn", C.c_int32),
                ("tokens", C.c_int32), ("fp_ns", C.c_uint64), ("bp_ns", C.c_uint64), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_uint64), ("seed", C.c_uint64)]


class fr_stage_desc(C.Structure):
    _fields_ = [("schedule", C.c_int32), ("p", C.c_int32), ("m", C.c_int32), ("stage", C.c_int32),
                ("f_ns", C.c_uint64), ("b_ns", C.c_uint64), ("chunks", C.c_int32), ("reserved", C.c_int32)]


class fr_stage_op(C.Structure):
    _fields_ = [("kind", C.c_int32), ("microbatch", C.c_int32), ("start_ns", C.c_uint64), ("end_ns", C.c_uint64),
                ("bubble_before_ns", C.c_uint64), ("chunk", C.c_int32), ("reserved", C.c_int32)]


class fr_epoch_result(C.Structure):
    _fields_ = [("epoch_ns", C.c_uint64), ("busy_ns", C.c_uint64), ("bubble_ns", C.c_uint64), ("n_ops", C.c_uint32),
                ("n_bubbles", C.c_uint32), ("overruns", C.c_uint32), ("reserved", C.c_uint32)]


# name -> (restype, argtypes); every symbol the header declares
SIGNATURES = {
    "fr_create": (C.c_int, [C.POINTER(fr_config), C.POINTER(C.c_void_p)]),
    "fr_destroy": (C.c_int, [C.c_void_p]),
    "fr_side_stream": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p)]),
    "fr_last_hip_error": (C.c_int, [C.c_void_p]),
    "fr_now_ns": (C.c_uint64, []),
    "fr_task_register": (C.c_int, [C.c_void_p, C.POINTER(fr_task_ops), C.c_void_p, C.POINTER(fr_task_profile), C.POINTER(C.c_int32)]),
    "fr_task_stop": (C.c_int, [C.c_void_p, C.c_int32]),
    "fr_alloc_device": (C.c_void_p, [C.c_void_p, C.c_size_t]),
    "fr_alloc_charge": (C.c_int, [C.c_void_p, C.c_size_t]),
    "fr_alloc_free": (C.c_int, [C.c_void_p, C.c_void_p]),
    "fr_alloc_used": (C.c_uint64, [C.c_void_p]),
    "fr_alloc_peak": (C.c_uint64, [C.c_void_p]),
    "fr_bubble_begin": (C.c_int, [C.c_void_p, C.c_uint64, C.c_uint64]),
    "fr_bubble_end": (C.c_int, [C.c_void_p]),
    "fr_query_progress": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(fr_progress)]),
    "fr_event_log": (C.c_int, [C.c_void_p, C.POINTER(fr_event), C.c_size_t, C.POINTER(C.c_size_t)]),
    "fr_event_log_clear": (C.c_int, [C.c_void_p]),
    "fr_chunk_fit": (C.c_int, [C.POINTER(C.c_uint64), C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint64, C.POINTER(C.c_uint32)]),
    "fr_cost_scale_next": (C.c_uint32, [C.c_uint32, C.c_uint64, C.c_uint64]),
    "fr_cost_scales": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint32)]),
    "fr_pagerank_make": (C.c_int, [C.POINTER(fr_pagerank_desc), C.POINTER(fr_task_ops), C.POINTER(C.c_void_p), C.POINTER(fr_task_profile)]),
    "fr_pagerank_destroy": (C.c_int, [C.c_void_p]),
    "fr_pagerank_info": (C.c_int, [C.c_void_p, C.POINTER(fr_pagerank_info_t)]),
    "fr_pagerank_tiles": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_uint32)]),
    "fr_pagerank_tile_costs": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_uint32), C.c_size_t, C.POINTER(C.c_size_t)]),
    "fr_pagerank_tile_work": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_uint64), C.c_size_t, C.POINTER(C.c_size_t)]),
    "fr_pagerank_tile_weights": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_uint64), C.c_size_t, C.POINTER(C.c_size_t)]),
    "fr_pagerank_run_standalone": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_uint32, C.POINTER(C.c_uint64)]),
    "fr_sgd_make": (C.c_int, [C.POINTER(fr_sgd_desc), C.POINTER(fr_task_ops), C.POINTER(C.c_void_p), C.POINTER(fr_task_profile)]),
    "fr_sgd_destroy": (C.c_int, [C.c_void_p]),
    "fr_sgd_info": (C.c_int, [C.c_void_p, C.POINTER(fr_sgd_info_t)]),
    "fr_sgd_block_starts": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_uint32), C.c_size_t, C.POINTER(C.c_size_t)]),
    "fr_sgd_cell_sizes": (C.c_int, [C.c_void_p, C.c_uint32, C.POINTER(C.c_uint32), C.c_size_t, C.POINTER(C.c_size_t)]),
    "fr_pagerank_run_standalone_noalloc": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_uint32]),
    "fr_sgd_run_standalone": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_uint32, C.POINTER(C.c_uint64)]),
    "fr_load_workspace_bytes": (C.c_int, [C.POINTER(fr_load_desc), C.POINTER(C.c_uint64)]),
    "fr_load_make": (C.c_int, [C.POINTER(fr_load_desc), C.c_void_p, C.POINTER(C.c_void_p)]),
    "fr_load_destroy": (C.c_int, [C.c_void_p]),
    "fr_load_fp": (C.c_int, [C.c_void_p, C.c_void_p]),
    "fr_load_bp": (C.c_int, [C.c_void_p, C.c_void_p]),
    "fr_load_part": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32]),
    "fr_load_flops": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]),
    "fr_gemm_bf16": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]),
    "fr_stage_make": (C.c_int, [C.POINTER(fr_stage_desc), C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]),
    "fr_stage_destroy": (C.c_int, [C.c_void_p]),
    "fr_stage_ops": (C.c_int, [C.c_void_p, C.POINTER(fr_stage_op), C.c_size_t, C.POINTER(C.c_size_t), C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]),
    "fr_stage_run_epoch": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(fr_epoch_result)]),
    "fr_stage_set_filler": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint64]),
    "fr_stage_op_times": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint64), C.c_size_t, C.POINTER(C.c_size_t)]),
}

_lib = None


def lib() -> C.CDLL:
    """The loaded library.  Builds it first only when no built library exists; never falls back to anything else."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            _build.build()
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)          # AttributeError here = the library does not export a declared symbol
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _check(code, where, allow=()):
    if code != FR_OK and code not in allow:
        raise FreeRideError(code, where)
    return code


def _ptr(x):
    """Device/host pointer from an int, a torch tensor (data_ptr) or a numpy array."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "ctypes"):
        return x.ctypes.data
    raise TypeError(type(x))


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return s.cuda_stream


def fr_now_ns():
    return lib().fr_now_ns()


def fr_chunk_fit(prefix, tile0, budget_ns, launch_cost_ns):
    n = len(prefix) - 1
    arr = (C.c_uint64 * (n + 1))(*prefix)
    out = C.c_uint32()
    _check(lib().fr_chunk_fit(arr, n, tile0, budget_ns, launch_cost_ns, C.byref(out)), "fr_chunk_fit")
    return out.value


def fr_cost_scale_next(scale_ppm, modelled_ns, measured_ns):
    return lib().fr_cost_scale_next(scale_ppm, modelled_ns, measured_ns)


class Context:
    """fr_ctx: one GPU, one stage."""

    def __init__(self, device_id=0, cu_count=0, cu_mask=None, mem_available_bytes=1 << 62, guard_ns=0,
                 launch_cost_ns=0, max_chunk_ns=0, max_inflight=0, event_log_capacity=0, time_steps=0, grace_ns=0,
                 adapt_costs=0, device_gate=0, gate_guard_ns=0):
        cfg = fr_config()
        cfg.device_id = device_id
        cfg.cu_count = cu_count
        for i, w in enumerate(cu_mask or []):
            cfg.cu_mask[i] = w
        cfg.mem_available_bytes = mem_available_bytes
        cfg.guard_ns, cfg.launch_cost_ns, cfg.max_chunk_ns = guard_ns, launch_cost_ns, max_chunk_ns
        cfg.max_inflight, cfg.event_log_capacity, cfg.time_steps = max_inflight, event_log_capacity, time_steps
        cfg.grace_ns, cfg.adapt_costs, cfg.device_gate = grace_ns, adapt_costs, device_gate
        cfg.gate_guard_ns = gate_guard_ns
        self.handle = C.c_void_p()
        _check(lib().fr_create(C.byref(cfg), C.byref(self.handle)), "fr_create")
        self._keep = []

    def fr_destroy(self):
        if self.handle:
            _check(lib().fr_destroy(self.handle), "fr_destroy")
            self.handle = C.c_void_p()

    def fr_side_stream(self):
        out = C.c_void_p()
        _check(lib().fr_side_stream(self.handle, C.byref(out)), "fr_side_stream")
        return out.value

    def fr_last_hip_error(self):
        return lib().fr_last_hip_error(self.handle)

    def fr_task_register(self, ops, user, profile):
        tid = C.c_int32()
        self._keep.append((ops, user, profile))
        _check(lib().fr_task_register(self.handle, C.byref(ops), user, C.byref(profile), C.byref(tid)), "fr_task_register")
        return tid.value

    def fr_task_stop(self, task_id):
        return _check(lib().fr_task_stop(self.handle, task_id), "fr_task_stop")

    def fr_bubble_begin(self, t_begin_ns, duration_ns):
        return _check(lib().fr_bubble_begin(self.handle, t_begin_ns, duration_ns), "fr_bubble_begin")

    def fr_bubble_end(self):
        """Returns FR_OK or FR_ERR_OVERRUN."""
        return _check(lib().fr_bubble_end(self.handle), "fr_bubble_end", allow=(FR_ERR_OVERRUN,))

    def fr_query_progress(self, task_id):
        out = fr_progress()
        _check(lib().fr_query_progress(self.handle, task_id, C.byref(out)), "fr_query_progress")
        return out

    def fr_event_log(self, cap=1 << 16):
        buf = (fr_event * cap)()
        n = C.c_size_t()
        _check(lib().fr_event_log(self.handle, buf, cap, C.byref(n)), "fr_event_log")
        return [buf[i] for i in range(n.value)]

    def fr_event_log_clear(self):
        return _check(lib().fr_event_log_clear(self.handle), "fr_event_log_clear")

    def fr_cost_scales(self):
        out = (C.c_uint32 * 8)()
        _check(lib().fr_cost_scales(self.handle, out), "fr_cost_scales")
        return list(out)


class PageRankTask:
    """fr_pagerank_make and friends.  Tensors (torch, on the GPU) are only read for their data_ptr."""

    def __init__(self, n_vertices, n_edges, row_ptr, col, out_degree, ranks_out, damping=0.85, iterations=30,
                 max_runs=0, mem_limit_bytes=1 << 40, fs_per_edge=0, fs_per_message=0, fs_per_vertex=0,
                 finish_tile_ns=0, min_step_ns=(0, 0, 0, 0), rows_per_partition=0, sources_per_partition=0):
        d = fr_pagerank_desc()
        d.n_vertices, d.n_edges = n_vertices, n_edges
        d.row_ptr, d.col, d.out_degree, d.ranks_out = _ptr(row_ptr), _ptr(col), _ptr(out_degree), _ptr(ranks_out)
        d.damping, d.iterations, d.max_runs = damping, iterations, max_runs
        d.mem_limit_bytes = mem_limit_bytes
        d.fs_per_edge, d.fs_per_message, d.fs_per_vertex = fs_per_edge, fs_per_message, fs_per_vertex
        d.finish_tile_ns = finish_tile_ns
        for k in range(4):
            d.min_step_ns[k] = int(min_step_ns[k])
        d.rows_per_partition, d.sources_per_partition = rows_per_partition, sources_per_partition
        self.desc = d
        self._keep = (row_ptr, col, out_degree, ranks_out)
        self.ops = fr_task_ops()
        self.user = C.c_void_p()
        self.profile = fr_task_profile()
        _check(lib().fr_pagerank_make(C.byref(d), C.byref(self.ops), C.byref(self.user), C.byref(self.profile)),
               "fr_pagerank_make")

    def fr_pagerank_destroy(self):
        if self.user:
            _check(lib().fr_pagerank_destroy(self.user), "fr_pagerank_destroy")
            self.user = C.c_void_p()

    def fr_pagerank_info(self):
        out = fr_pagerank_info_t()
        _check(lib().fr_pagerank_info(self.user, C.byref(out)), "fr_pagerank_info")
        return out

    def fr_pagerank_tile_work(self, seg_kind):
        n = self.fr_pagerank_tiles(seg_kind)
        buf = (C.c_uint64 * n)()
        got = C.c_size_t()
        _check(lib().fr_pagerank_tile_work(self.user, seg_kind, buf, n, C.byref(got)), "fr_pagerank_tile_work")
        return list(buf)

    def fr_pagerank_tile_weights(self, seg_kind):
        n = self.fr_pagerank_tiles(seg_kind)
        buf = (C.c_uint64 * n)()
        got = C.c_size_t()
        _check(lib().fr_pagerank_tile_weights(self.user, seg_kind, buf, n, C.byref(got)), "fr_pagerank_tile_weights")
        return list(buf)

    def fr_pagerank_tiles(self, seg_kind):
        out = C.c_uint32()
        _check(lib().fr_pagerank_tiles(self.user, seg_kind, C.byref(out)), "fr_pagerank_tiles")
        return out.value

    def fr_pagerank_tile_costs(self, seg_kind):
        n = self.fr_pagerank_tiles(seg_kind)
        buf = (C.c_uint32 * n)()
        got = C.c_size_t()
        _check(lib().fr_pagerank_tile_costs(self.user, seg_kind, buf, n, C.byref(got)), "fr_pagerank_tile_costs")
        return list(buf)

    def fr_pagerank_run_standalone(self, device_id=0, stream=None, max_tiles_per_launch=0, want_phase_ns=False):
        ph = (C.c_uint64 * 4)()
        _check(lib().fr_pagerank_run_standalone(self.user, device_id, _stream(stream), max_tiles_per_launch,
                                                ph if want_phase_ns else None), "fr_pagerank_run_standalone")
        return list(ph) if want_phase_ns else None

    def fr_pagerank_run_standalone_noalloc(self, device_id=0, stream=None, max_tiles_per_launch=0):
        _check(lib().fr_pagerank_run_standalone_noalloc(self.user, device_id, _stream(stream), max_tiles_per_launch),
               "fr_pagerank_run_standalone_noalloc")


class SgdTask:
    """fr_sgd_make and friends.  Tensors (torch, on the GPU) are only read for their data_ptr."""

    def __init__(self, n_users, n_items, n_ratings, row_ptr, item, rating, P, Q, factors, gamma, lam, iterations=1,
                 blocks=0, max_runs=0, mem_limit_bytes=1 << 40, fs_per_rating=0, min_step_ns=0, fs_per_chain_rating=0):
        d = fr_sgd_desc()
        d.n_users, d.n_items, d.n_ratings = n_users, n_items, n_ratings
        d.row_ptr, d.item, d.rating, d.P, d.Q = _ptr(row_ptr), _ptr(item), _ptr(rating), _ptr(P), _ptr(Q)
        d.factors, d.blocks, d.gamma, d.lam = factors, blocks, gamma, lam
        d.iterations, d.max_runs, d.mem_limit_bytes = iterations, max_runs, mem_limit_bytes
        d.fs_per_rating, d.min_step_ns, d.fs_per_chain_rating = fs_per_rating, min_step_ns, fs_per_chain_rating
        self.desc = d
        self._keep = (row_ptr, item, rating, P, Q)
        self.ops = fr_task_ops()
        self.user = C.c_void_p()
        self.profile = fr_task_profile()
        _check(lib().fr_sgd_make(C.byref(d), C.byref(self.ops), C.byref(self.user), C.byref(self.profile)), "fr_sgd_make")

    def fr_sgd_destroy(self):
        if self.user:
            _check(lib().fr_sgd_destroy(self.user), "fr_sgd_destroy")
            self.user = C.c_void_p()

    def fr_sgd_info(self):
        out = fr_sgd_info_t()
        _check(lib().fr_sgd_info(self.user, C.byref(out)), "fr_sgd_info")
        return out

    def fr_sgd_block_starts(self, items):
        n = self.fr_sgd_info().blocks + 1
        buf = (C.c_uint32 * n)()
        got = C.c_size_t()
        _check(lib().fr_sgd_block_starts(self.user, 1 if items else 0, buf, n, C.byref(got)), "fr_sgd_block_starts")
        return list(buf)

    def fr_sgd_cell_sizes(self, stratum):
        n = self.fr_sgd_info().blocks
        buf = (C.c_uint32 * n)()
        got = C.c_size_t()
        _check(lib().fr_sgd_cell_sizes(self.user, stratum, buf, n, C.byref(got)), "fr_sgd_cell_sizes")
        return list(buf)

    def fr_sgd_run_standalone(self, device_id=0, stream=None, max_cells_per_launch=0, want_ns=False):
        ns = C.c_uint64()
        _check(lib().fr_sgd_run_standalone(self.user, device_id, _stream(stream), max_cells_per_launch,
                                           C.byref(ns) if want_ns else None), "fr_sgd_run_standalone")
        return ns.value if want_ns else None


class Load:
    """fr_load: busy-wait or GPT-shaped GEMM bursts."""

    def __init__(self, kind, layers=0, hidden=0, ffn=0, tokens=0, fp_ns=0, bp_ns=0, workspace=None, seed=0, stream=None):
        d = fr_load_desc()
        d.kind, d.layers, d.hidden, d.ffn, d.tokens = kind, layers, hidden, ffn, tokens
        d.fp_ns, d.bp_ns, d.seed = fp_ns, bp_ns, seed
        d.workspace = _ptr(workspace)
        d.workspace_bytes = (workspace.numel() * workspace.element_size()) if workspace is not None else 0
        self._keep = workspace
        self.handle = C.c_void_p()
        _check(lib().fr_load_make(C.byref(d), _stream(stream), C.byref(self.handle)), "fr_load_make")

    @staticmethod
    def fr_load_workspace_bytes(kind, layers=0, hidden=0, ffn=0, tokens=0):
        d = fr_load_desc()
        d.kind, d.layers, d.hidden, d.ffn, d.tokens = kind, layers, hidden, ffn, tokens
        out = C.c_uint64()
        _check(lib().fr_load_workspace_bytes(C.byref(d), C.byref(out)), "fr_load_workspace_bytes")
        return out.value

    def fr_load_fp(self, stream=None):
        return _check(lib().fr_load_fp(self.handle, _stream(stream)), "fr_load_fp")

    def fr_load_bp(self, stream=None):
        return _check(lib().fr_load_bp(self.handle, _stream(stream)), "fr_load_bp")

    def fr_load_part(self, stream=None, kind=0, part=0, parts=1):
        return _check(lib().fr_load_part(self.handle, _stream(stream), kind, part, parts), "fr_load_part")

    def fr_load_flops(self):
        a, b = C.c_uint64(), C.c_uint64()
        _check(lib().fr_load_flops(self.handle, C.byref(a), C.byref(b)), "fr_load_flops")
        return a.value, b.value

    def fr_load_destroy(self):
        if self.handle:
            _check(lib().fr_load_destroy(self.handle), "fr_load_destroy")
            self.handle = C.c_void_p()


def fr_gemm_bf16(A, B, Cmat, M, N, K, stream=None):
    return _check(lib().fr_gemm_bf16(_ptr(A), _ptr(B), _ptr(Cmat), M, N, K, _stream(stream)), "fr_gemm_bf16")


class Stage:
    """fr_stage: one emulated pipeline stage."""

    def __init__(self, schedule, p, m, stage, f_ns, b_ns, load=None, stream=None, chunks=0):
        d = fr_stage_desc()
        d.schedule, d.p, d.m, d.stage, d.f_ns, d.b_ns, d.chunks = schedule, p, m, stage, f_ns, b_ns, chunks
        self._keep = (load, stream)
        self.handle = C.c_void_p()
        _check(lib().fr_stage_make(C.byref(d), load.handle if load is not None else None, _stream(stream),
                                   C.byref(self.handle)), "fr_stage_make")

    def fr_stage_ops(self):
        n = C.c_size_t()
        epoch, tail = C.c_uint64(), C.c_uint64()
        _check(lib().fr_stage_ops(self.handle, None, 0, C.byref(n), C.byref(epoch), C.byref(tail)), "fr_stage_ops")
        buf = (fr_stage_op * n.value)()
        _check(lib().fr_stage_ops(self.handle, buf, n.value, C.byref(n), C.byref(epoch), C.byref(tail)), "fr_stage_ops")
        return [buf[i] for i in range(n.value)], epoch.value, tail.value

    def fr_stage_run_epoch(self, ctx=None):
        out = fr_epoch_result()
        _check(lib().fr_stage_run_epoch(self.handle, ctx.handle if ctx is not None else None, C.byref(out)),
               "fr_stage_run_epoch")
        return out

    def fr_stage_set_filler(self, stream=None, workgroups=0, guard_ns=0):
        _check(lib().fr_stage_set_filler(self.handle, _stream(stream), workgroups, guard_ns), "fr_stage_set_filler")

    def fr_stage_op_times(self):
        n = C.c_size_t()
        _check(lib().fr_stage_op_times(self.handle, None, 0, C.byref(n)), "fr_stage_op_times")
        buf = (C.c_uint64 * max(1, n.value))()
        _check(lib().fr_stage_op_times(self.handle, buf, n.value, C.byref(n)), "fr_stage_op_times")
        return list(buf)[:n.value]

    def fr_stage_destroy(self):
        if self.handle:
            _check(lib().fr_stage_destroy(self.handle), "fr_stage_destroy")
            self.handle = C.c_void_p()
