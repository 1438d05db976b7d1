"""ctypes binding of include/cacheflow.h.  Argument marshalling only: names,
argument order and meaning follow the C header one to one."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcacheflow.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is not built; run `python -m paper_2604_25080_amd.build` "
        "(there is no fallback path)")
lib = C.CDLL(LIB_PATH)

CF_OK = 0
CF_ERR_INVALID_ARG, CF_ERR_INVALID_PLAN, CF_ERR_OUT_OF_PAGES, CF_ERR_HIP = -1, -2, -3, -4
CF_ERR_UNKNOWN_REQUEST, CF_ERR_WORKSPACE, CF_ERR_UNSUPPORTED = -5, -6, -7
CF_F32, CF_BF16 = 0, 1
CF_TOKEN_WISE, CF_LAYER_WISE = 0, 1
CF_KEY_REMAINING_COST, CF_KEY_REMAINING_CELLS, CF_KEY_MARGINAL = 0, 1, 2
EPI_STORE_F32, EPI_ADD_F32, EPI_STORE_T, EPI_SILU_MUL = 0, 1, 2, 3
PAGE_TOKENS = 16


class CfError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib.cf_last_error().decode()
        super().__init__(f"{where}: {lib.cf_status_str(status).decode()} ({status}): {msg}")


class cf_cost_model(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("f_c", "alpha", "beta", "f_io", "gamma", "s_c", "s_io")]


class cf_plan_opts(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("chunk_tokens", "l_delta", "n_layers",
                                         "kv_bytes_per_token_layer", "force_mode", "io_key",
                                         "kv_only_permille", "boundary_bytes_per_token")]


class cf_split(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("mode", "k_tokens", "layer_cut")]


class cf_claim(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("engine", "request", "unit")]


class cf_plan_stats(C.Structure):
    _fields_ = [("t_comp", C.c_int64), ("t_io", C.c_int64), ("makespan", C.c_int64),
                ("n_claims", C.c_int32), ("n_trace", C.c_int32)]


class cf_model_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads",
                                         "head_dim", "d_ffn", "vocab", "dtype")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float)]


class cf_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wqkv", "wo", "mlp_norm", "w_gate",
                                          "w_up", "w_down")]


class cf_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("layers", C.POINTER(cf_layer_weights))]


class cf_ctx_opts(C.Structure):
    _fields_ = [("max_batch", C.c_int32), ("max_tokens", C.c_int32), ("max_positions", C.c_int32),
                ("chunk_rows", C.c_int32), ("staging_bytes", C.c_int64)]


class cf_request(C.Structure):
    _fields_ = [("req_id", C.c_uint64), ("ctx_tokens", C.c_void_p), ("n_ctx", C.c_int32),
                ("n_new", C.c_int32), ("host_kv", C.c_void_p), ("new_tokens", C.c_void_p),
                ("boundary_h", C.c_void_p)]


class cf_timing(C.Structure):
    _fields_ = [("restore_ms", C.c_float), ("compute_ms", C.c_float), ("copy_ms", C.c_float),
                ("suffix_ms", C.c_float), ("total_ms", C.c_float), ("compute_wait_ms", C.c_float),
                ("recompute_flops", C.c_double), ("suffix_flops", C.c_double),
                ("loaded_bytes", C.c_int64), ("recomputed_cells", C.c_int64),
                ("loaded_cells", C.c_int64)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class cf_dynamic_stats(C.Structure):
    _fields_ = [("compute_steps", C.c_int32), ("compute_units", C.c_int32), ("io_units", C.c_int32),
                ("scale_c_permille", C.c_int32), ("scale_io_permille", C.c_int32),
                ("scale_io_alone_permille", C.c_int32), ("planned_tail", C.c_int32),
                ("last_step_merged", C.c_int32), ("compute_gap_ms", C.c_double)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class cf_overlap_model(C.Structure):
    _fields_ = [("comp_permille", C.c_int32), ("io_permille", C.c_int32)]


class cf_batch_plan_opts(C.Structure):
    _fields_ = [("chunk_tokens", C.c_int32), ("l_delta", C.c_int32), ("force_mode", C.c_int32),
                ("io_key", C.c_int32), ("pipelined_join", C.c_int32), ("stage_layers", C.c_int32),
                ("stage_first_layer", C.c_int32)]


class cf_batch_plan(C.Structure):
    _fields_ = [("kind", C.c_int32), ("kv_only_permille", C.c_int32), ("pipelined_join", C.c_int32),
                ("reserved", C.c_int32), ("prefill_ps", C.c_int64), ("t_comp", C.c_int64), ("t_io", C.c_int64),
                ("ttft", C.c_int64), ("ttft_hybrid", C.c_int64), ("ttft_all_load", C.c_int64),
                ("ttft_all_recompute", C.c_int64)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


PLAN_HYBRID, PLAN_ALL_LOAD, PLAN_ALL_RECOMPUTE = 0, 1, 2


class cf_dynamic_opts(C.Structure):
    _fields_ = [("step_cap_ps", C.c_int64), ("order", C.c_int32), ("units_per_request", C.c_int32),
                ("overlap_comp_permille", C.c_int32), ("overlap_io_permille", C.c_int32)]


ORDER_CHEAPEST, ORDER_SHORTEST = 0, 1


class cf_kernel_stat(C.Structure):
    _fields_ = [("kernel", C.c_int32), ("launches", C.c_int32), ("total_ms", C.c_double),
                ("work", C.c_double)]


KERNEL_NAMES = ["gemm_qkv", "gemm_oproj", "gemm_gate_up", "gemm_down", "gemm_lm_head", "attention",
                "rmsnorm", "rope_write", "embed", "page_scatter", "h2d_copy"]
CF_N_KERNELS = len(KERNEL_NAMES)

_P = C.POINTER
lib.cf_status_str.restype = C.c_char_p
lib.cf_status_str.argtypes = [C.c_int]
lib.cf_last_error.restype = C.c_char_p
lib.cf_last_error.argtypes = []
lib.cf_restore_plan.argtypes = [_P(cf_cost_model), _P(cf_plan_opts), C.c_int32, C.c_void_p,
                                _P(cf_split), _P(cf_plan_stats), _P(cf_claim), C.c_int32]
lib.cf_plan_eval.argtypes = [_P(cf_cost_model), _P(cf_plan_opts), C.c_int32, C.c_void_p,
                             _P(cf_split), _P(C.c_int64), _P(C.c_int64)]
lib.cf_cost_feedback.argtypes = [_P(cf_cost_model), C.c_int64, C.c_int64, C.c_int64, C.c_int64]
lib.cf_prefill_cost.argtypes = [_P(cf_cost_model), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                _P(C.c_int64)]
lib.cf_plan_batch.argtypes = [_P(cf_cost_model), _P(cf_overlap_model), _P(cf_model_desc), _P(cf_batch_plan_opts),
                              C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, _P(cf_batch_plan)]
lib.cf_plan_feedback.argtypes = [_P(cf_cost_model), _P(cf_overlap_model), _P(cf_batch_plan), C.c_int64,
                                 C.c_int64, C.c_int64, C.c_int64]
lib.cf_calibrate_overlap.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, _P(cf_cost_model),
                                     _P(cf_overlap_model)]
lib.cf_derive_l_delta.argtypes = [_P(cf_cost_model), _P(cf_plan_opts), C.c_int32, _P(C.c_int32)]
lib.cf_dynamic_io_pick.argtypes = [_P(cf_cost_model), _P(cf_plan_opts), C.c_int32, C.c_void_p,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                   C.c_int32, C.c_int32, _P(C.c_int32)]
lib.cf_dynamic_claim.argtypes = [_P(cf_cost_model), _P(cf_plan_opts), C.c_int32, C.c_void_p,
                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                 C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                 C.c_int32, C.c_int32, C.c_void_p, _P(C.c_int64)]
lib.cf_cache_create.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                _P(C.c_void_p)]
lib.cf_cache_destroy.argtypes = [C.c_void_p]
lib.cf_cache_destroy.restype = None
lib.cf_cache_n_pages.argtypes = [C.c_void_p]
lib.cf_cache_n_free.argtypes = [C.c_void_p]
lib.cf_cache_page_bytes.argtypes = [C.c_void_p]
lib.cf_cache_page_bytes.restype = C.c_size_t
lib.cf_cache_alloc.argtypes = [C.c_void_p, C.c_uint64, C.c_int32]
lib.cf_cache_free.argtypes = [C.c_void_p, C.c_uint64]
lib.cf_cache_page_table.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_int32, _P(C.c_int32)]
lib.cf_host_kv_bytes.argtypes = [C.c_int32] * 5
lib.cf_host_kv_bytes.restype = C.c_size_t
lib.cf_workspace_bytes.argtypes = [_P(cf_model_desc), _P(cf_ctx_opts), _P(C.c_size_t)]
lib.cf_ctx_create.argtypes = [_P(cf_model_desc), _P(cf_weights), _P(cf_ctx_opts), C.c_void_p,
                              C.c_size_t, C.c_void_p, C.c_void_p, _P(C.c_void_p)]
lib.cf_ctx_destroy.argtypes = [C.c_void_p]
lib.cf_ctx_destroy.restype = None
lib.cf_ctx_set_kernel_set.argtypes = [C.c_void_p, C.c_int32]
lib.cf_ctx_set_pipelined_join.argtypes = [C.c_void_p, C.c_int32]
lib.cf_ctx_set_load_path.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
lib.cf_ctx_set_link_throttle.argtypes = [C.c_void_p, C.c_double]
lib.cf_ctx_set_stage.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
lib.cf_ctx_capture_boundary.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int64]
lib.cf_ctx_capture_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
lib.cf_restore_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, _P(cf_request), _P(cf_split),
                                 C.c_void_p, _P(cf_timing)]
lib.cf_restore_dynamic.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, _P(cf_request),
                                   _P(cf_cost_model), _P(cf_plan_opts), _P(cf_dynamic_opts),
                                   C.c_void_p, _P(cf_split), _P(cf_timing), _P(cf_dynamic_stats)]
lib.cf_offload.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_int32, C.c_void_p]
lib.cf_offload_static.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_int32, C.c_void_p]
lib.cf_offload_static_max_tokens.restype = C.c_size_t
lib.cf_offload_static_max_tokens.argtypes = []
lib.cf_ctx_inject_failure.argtypes = [C.c_void_p, C.c_int32]
lib.cf_debug_force_gemm_tile.argtypes = [C.c_int32]
lib.cf_measure_h2d.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32,
                               _P(C.c_double)]
lib.cf_calibrate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, _P(cf_cost_model)]
lib.cf_ctx_profile.argtypes = [C.c_void_p, C.c_uint32]
lib.cf_ctx_profile_read.argtypes = [C.c_void_p, _P(cf_kernel_stat), C.c_int32]
lib.cf_read_final_hidden.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
lib.cf_op_gemm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                           C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                           _P(C.c_float)]

EXPORTS = ["cf_status_str", "cf_last_error", "cf_restore_plan", "cf_plan_eval", "cf_cost_feedback", "cf_prefill_cost",
           "cf_plan_batch", "cf_plan_feedback", "cf_calibrate_overlap",
           "cf_derive_l_delta", "cf_dynamic_io_pick", "cf_dynamic_claim", "cf_restore_dynamic", "cf_cache_create", "cf_cache_destroy", "cf_cache_n_pages",
           "cf_cache_n_free", "cf_cache_page_bytes", "cf_cache_alloc", "cf_cache_free",
           "cf_cache_page_table", "cf_host_kv_bytes", "cf_workspace_bytes", "cf_ctx_create",
           "cf_ctx_destroy", "cf_ctx_set_kernel_set", "cf_ctx_set_pipelined_join", "cf_ctx_set_load_path", "cf_ctx_set_link_throttle", "cf_ctx_set_stage", "cf_ctx_capture_boundary", "cf_ctx_capture_rows", "cf_restore_batch", "cf_offload",
           "cf_offload_static", "cf_offload_static_max_tokens", "cf_ctx_inject_failure", "cf_debug_force_gemm_tile",
           "cf_measure_h2d", "cf_op_gemm", "cf_calibrate", "cf_ctx_profile",
           "cf_ctx_profile_read", "cf_read_final_hidden"]


def _check(status, where):
    if status != CF_OK:
        raise CfError(status, where)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


# ------------------------------------------------------------------- planner
def cost_model(f_c, alpha, beta, f_io, gamma, s_c=0, s_io=0):
    return cf_cost_model(int(f_c), int(alpha), int(beta), int(f_io), int(gamma), int(s_c),
                         int(s_io))


def plan_opts(chunk_tokens, l_delta, n_layers, kv_bytes_per_token_layer, force_mode=-1,
              io_key=CF_KEY_REMAINING_COST, kv_only_permille=0, boundary_bytes_per_token=0):
    return cf_plan_opts(chunk_tokens, l_delta, n_layers, kv_bytes_per_token_layer, force_mode,
                        io_key, kv_only_permille, boundary_bytes_per_token)


def restore_plan(cost, opts, n_ctx, trace_cap=0):
    """-> (splits [(mode,k,cut)], stats dict, trace [(engine,request,unit)])"""
    n = _i32(n_ctx)
    b = len(n)
    splits = (cf_split * max(b, 1))()
    stats = cf_plan_stats()
    trace = (cf_claim * max(trace_cap, 1))()
    _check(lib.cf_restore_plan(C.byref(cost), C.byref(opts), b, n.ctypes.data, splits,
                               C.byref(stats), trace if trace_cap else None, trace_cap),
           "cf_restore_plan")
    out = [(splits[i].mode, splits[i].k_tokens, splits[i].layer_cut) for i in range(b)]
    st = dict(t_comp=stats.t_comp, t_io=stats.t_io, makespan=stats.makespan,
              n_claims=stats.n_claims)
    tr = [(trace[i].engine, trace[i].request, trace[i].unit) for i in range(stats.n_trace)]
    return out, st, tr


def overlap_model(comp_permille=1000, io_permille=1000):
    return cf_overlap_model(int(comp_permille), int(io_permille))


def batch_plan_opts(chunk_tokens, l_delta, force_mode=-1, io_key=0, pipelined_join=True, stage_layers=0,
                    stage_first_layer=0):
    return cf_batch_plan_opts(int(chunk_tokens), int(l_delta), int(force_mode), int(io_key),
                              int(bool(pipelined_join)), int(stage_layers), int(stage_first_layer))


def plan_batch(cost, overlap, desc, opts, n_ctx, n_new=None):
    """-> (splits [(mode,k,cut)], cf_batch_plan): the planning policy around Algorithm 1."""
    n = _i32(n_ctx)
    m = _i32(n_new) if n_new is not None else None
    b = len(n)
    splits = (cf_split * max(b, 1))()
    info = cf_batch_plan()
    _check(lib.cf_plan_batch(C.byref(cost), C.byref(overlap), C.byref(desc), C.byref(opts), b, n.ctypes.data,
                             m.ctypes.data if m is not None else None, splits, C.byref(info)), "cf_plan_batch")
    return [(splits[i].mode, splits[i].k_tokens, splits[i].layer_cut) for i in range(b)], info


def plan_feedback(cost, overlap, info, timing):
    """Closed loop after a batch (modifies cost / overlap in place).  timing: the dict returned by
    restore_batch (milliseconds -> picoseconds is the only conversion made here)."""
    ps = lambda ms: int(round(ms * 1e9))
    _check(lib.cf_plan_feedback(C.byref(cost), C.byref(overlap), C.byref(info), ps(timing["compute_ms"]),
                                ps(timing["copy_ms"]), ps(timing["total_ms"]), ps(timing["compute_wait_ms"])),
           "cf_plan_feedback")


def plan_eval(cost, opts, n_ctx, splits):
    n = _i32(n_ctx)
    arr = (cf_split * max(len(n), 1))(*[cf_split(*s) for s in splits])
    tc, tio = C.c_int64(), C.c_int64()
    _check(lib.cf_plan_eval(C.byref(cost), C.byref(opts), len(n), n.ctypes.data, arr,
                            C.byref(tc), C.byref(tio)), "cf_plan_eval")
    return tc.value, tio.value


def prefill_cost(cost, n_layers, n_ctx, n_new):
    """Compute-clock cost (ps) of the new-turn prefill of a batch under the cost model."""
    a = np.ascontiguousarray(n_ctx, dtype=np.int32)
    b = np.ascontiguousarray(n_new, dtype=np.int32)
    out = C.c_int64()
    _check(lib.cf_prefill_cost(C.byref(cost), int(n_layers), len(a), a.ctypes.data, b.ctypes.data,
                               C.byref(out)), "cf_prefill_cost")
    return out.value


def cost_feedback(cost, pred_comp, meas_comp, pred_io, meas_io):
    """Updates `cost` in place."""
    _check(lib.cf_cost_feedback(C.byref(cost), int(pred_comp), int(meas_comp), int(pred_io),
                                int(meas_io)), "cf_cost_feedback")
    return cost


def derive_l_delta(cost, opts, n_max):
    out = C.c_int32()
    _check(lib.cf_derive_l_delta(C.byref(cost), C.byref(opts), n_max, C.byref(out)),
           "cf_derive_l_delta")
    return out.value


def _closed(closed, b):
    arr = np.zeros(max(b, 1), dtype=np.uint8)
    if closed is not None:
        arr[:b] = np.asarray(closed, dtype=np.uint8)
    return arr


def dynamic_io_pick(cost, opts, n_ctx, p_comp, p_io, closed=None, io_backlog_ps=0,
                    compute_busy_ps=0, scale_c_permille=1000, scale_io_permille=1000):
    """Request whose far-end unit the I/O channel loads next, or -1."""
    n, pc, pio = _i32(n_ctx), _i32(p_comp), _i32(p_io)
    cl = _closed(closed, len(n))
    out = C.c_int32()
    _check(lib.cf_dynamic_io_pick(C.byref(cost), C.byref(opts), len(n), n.ctypes.data,
                                  pc.ctypes.data, pio.ctypes.data, cl.ctypes.data,
                                  int(io_backlog_ps), int(compute_busy_ps), int(scale_c_permille),
                                  int(scale_io_permille), C.byref(out)), "cf_dynamic_io_pick")
    return out.value


def dynamic_claim(cost, opts, n_ctx, p_comp, p_io, closed=None, io_backlog_ps=0,
                  scale_c_permille=1000, scale_io_permille=1000, step_fixed_ps=0, step_cap_ps=0,
                  order=0, compute_later_ps=0, max_units=1, io_alone_permille=0):
    """-> (take list, predicted step ps)"""
    n, pc, pio = _i32(n_ctx), _i32(p_comp), _i32(p_io)
    cl = _closed(closed, len(n))
    take = np.zeros(max(len(n), 1), dtype=np.int32)
    ps = C.c_int64()
    _check(lib.cf_dynamic_claim(C.byref(cost), C.byref(opts), len(n), n.ctypes.data, pc.ctypes.data,
                                pio.ctypes.data, cl.ctypes.data, int(io_backlog_ps),
                                int(step_fixed_ps), int(compute_later_ps), int(step_cap_ps), int(order),
                                int(scale_c_permille), int(scale_io_permille), int(max_units),
                                int(io_alone_permille), take.ctypes.data, C.byref(ps)), "cf_dynamic_claim")
    return [int(t) for t in take[:len(n)]], ps.value


# ---------------------------------------------------------------- page table
class Cache:
    """cf_cache handle.  `pool_ptr` is a device address (int) or 0."""

    def __init__(self, pool_ptr, pool_bytes, n_layers, n_kv_heads, head_dim, dtype):
        h = C.c_void_p()
        _check(lib.cf_cache_create(pool_ptr or None, pool_bytes, n_layers, n_kv_heads, head_dim,
                                   dtype, C.byref(h)), "cf_cache_create")
        self.handle = h

    def close(self):
        if self.handle and lib is not None:
            lib.cf_cache_destroy(self.handle)
            self.handle = None

    def __del__(self):
        self.close()

    @property
    def n_pages(self):
        return lib.cf_cache_n_pages(self.handle)

    @property
    def n_free(self):
        return lib.cf_cache_n_free(self.handle)

    @property
    def page_bytes(self):
        return lib.cf_cache_page_bytes(self.handle)

    def alloc(self, req_id, n_tokens):
        _check(lib.cf_cache_alloc(self.handle, req_id, n_tokens), "cf_cache_alloc")

    def free(self, req_id):
        _check(lib.cf_cache_free(self.handle, req_id), "cf_cache_free")

    def page_table(self, req_id):
        n = C.c_int32()
        _check(lib.cf_cache_page_table(self.handle, req_id, None, 0, C.byref(n)),
               "cf_cache_page_table")
        out = np.zeros(max(n.value, 1), dtype=np.int32)
        _check(lib.cf_cache_page_table(self.handle, req_id, out.ctypes.data, n.value,
                                       C.byref(n)), "cf_cache_page_table")
        return out[:n.value].tolist()


def host_kv_bytes(n_layers, n_kv_heads, head_dim, dtype, n_ctx):
    return lib.cf_host_kv_bytes(n_layers, n_kv_heads, head_dim, dtype, n_ctx)


# ------------------------------------------------------------------ executor
def model_desc(shape):
    """cf_model_desc from any object with the ModelShape fields."""
    return cf_model_desc(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads,
                         shape.head_dim, shape.d_ffn, shape.vocab,
                         CF_F32 if shape.dtype == "f32" else CF_BF16,
                         shape.rope_base, shape.rms_eps)


def ctx_opts(max_batch, max_tokens, max_positions, chunk_rows=0, staging_bytes=0):
    return cf_ctx_opts(max_batch, max_tokens, max_positions, chunk_rows, staging_bytes)


def workspace_bytes(desc, opts):
    n = C.c_size_t()
    _check(lib.cf_workspace_bytes(C.byref(desc), C.byref(opts), C.byref(n)), "cf_workspace_bytes")
    return n.value


class Ctx:
    """cf_ctx handle.  `weights` = dict(embed=ptr, lm_head=ptr, final_norm=ptr,
    layers=[dict(attn_norm=ptr, wqkv=ptr, ...)]) of device addresses (ints)."""

    def __init__(self, desc, weights, opts, workspace_ptr, workspace_bytes_, compute_stream,
                 copy_stream):
        layers = (cf_layer_weights * desc.n_layers)(*[
            cf_layer_weights(*[lw[n] for n, _ in cf_layer_weights._fields_])
            for lw in weights["layers"]])
        w = cf_weights(weights["embed"], weights["lm_head"], weights["final_norm"], layers)
        h = C.c_void_p()
        _check(lib.cf_ctx_create(C.byref(desc), C.byref(w), C.byref(opts), workspace_ptr,
                                 workspace_bytes_, compute_stream, copy_stream, C.byref(h)),
               "cf_ctx_create")
        self.handle = h
        self.desc = desc

    def close(self):
        if self.handle and lib is not None:
            lib.cf_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        self.close()

    def set_kernel_set(self, simple_only):
        _check(lib.cf_ctx_set_kernel_set(self.handle, int(simple_only)), "cf_ctx_set_kernel_set")

    def set_pipelined_join(self, on):
        _check(lib.cf_ctx_set_pipelined_join(self.handle, int(on)), "cf_ctx_set_pipelined_join")

    def set_load_path(self, path, n_workgroups=0):
        """path: 0 auto, 1 staged DMA + scatter, 2 direct load kernel."""
        _check(lib.cf_ctx_set_load_path(self.handle, int(path), int(n_workgroups)), "cf_ctx_set_load_path")

    def set_stage(self, layer_begin, layer_end):
        """Restrict restore_batch to layers [layer_begin, layer_end) (one pipeline stage)."""
        _check(lib.cf_ctx_set_stage(self.handle, int(layer_begin), int(layer_end)), "cf_ctx_set_stage")

    def capture_boundary(self, layer, dev_ptr, cap_rows):
        """One shot: the next restore_batch copies the rows entering `layer` to dev_ptr (float[cap_rows][d])."""
        _check(lib.cf_ctx_capture_boundary(self.handle, int(layer), dev_ptr, int(cap_rows)),
               "cf_ctx_capture_boundary")

    def capture_rows(self, packed_rows, dev_ptr):
        """One shot: the next restore_batch samples the residual stream of the listed packed rows
        into dev_ptr (float[2L+1][n_rows][d]): slot 2l = entering layer l, 2l+1 = entering its MLP
        half, 2L = leaving the last layer."""
        rows = _i32(packed_rows)
        _check(lib.cf_ctx_capture_rows(self.handle, rows.ctypes.data, len(rows), dev_ptr), "cf_ctx_capture_rows")

    def set_link_throttle(self, gb_per_s):
        """Pace the copy stream to gb_per_s GB/s (0: off)."""
        _check(lib.cf_ctx_set_link_throttle(self.handle, float(gb_per_s)), "cf_ctx_set_link_throttle")

    def restore_batch(self, cache, requests, splits, logits_ptr):
        """requests: list of dict(req_id, ctx_tokens (np.int32), n_new, host_kv (address or
        0), new_tokens (np.int32)); splits: [(mode,k,cut)].  Returns the timing dict."""
        b = len(requests)
        keep = []
        arr = (cf_request * max(b, 1))()
        for i, r in enumerate(requests):
            ct = _i32(r["ctx_tokens"])
            nt = _i32(r["new_tokens"])
            keep += [ct, nt]
            arr[i] = cf_request(r["req_id"], ct.ctypes.data if len(ct) else None, len(ct),
                                len(nt), r.get("host_kv") or None,
                                nt.ctypes.data if len(nt) else None, r.get("boundary_h") or None)
        sp = (cf_split * max(b, 1))(*[cf_split(*s) for s in splits])
        tm = cf_timing()
        _check(lib.cf_restore_batch(self.handle, cache.handle, b, arr, sp, logits_ptr or None,
                                    C.byref(tm)), "cf_restore_batch")
        return tm.as_dict()

    def restore_dynamic(self, cache, requests, cost, opts, logits_ptr, step_cap_ps=0,
                        order=ORDER_CHEAPEST, units_per_request=0, overlap=None):
        """Run-time scheduled restore.  Returns (splits [(mode,k,cut)], timing dict, stats dict)."""
        b = len(requests)
        keep = []
        arr = (cf_request * max(b, 1))()
        for i, r in enumerate(requests):
            ct = _i32(r["ctx_tokens"])
            nt = _i32(r["new_tokens"])
            keep += [ct, nt]
            arr[i] = cf_request(r["req_id"], ct.ctypes.data if len(ct) else None, len(ct),
                                len(nt), r.get("host_kv") or None,
                                nt.ctypes.data if len(nt) else None, None)
        sp = (cf_split * max(b, 1))()
        tm = cf_timing()
        st = cf_dynamic_stats()
        dyn = cf_dynamic_opts(int(step_cap_ps), int(order), int(units_per_request),
                              overlap.comp_permille if overlap is not None else 0,
                              overlap.io_permille if overlap is not None else 0)
        _check(lib.cf_restore_dynamic(self.handle, cache.handle, b, arr, C.byref(cost), C.byref(opts),
                                      C.byref(dyn), logits_ptr or None, sp, C.byref(tm), C.byref(st)),
               "cf_restore_dynamic")
        return ([(sp[i].mode, sp[i].k_tokens, sp[i].layer_cut) for i in range(b)], tm.as_dict(),
                st.as_dict())

    def offload(self, cache, req_id, n_ctx, host_ptr):
        _check(lib.cf_offload(self.handle, cache.handle, req_id, n_ctx, host_ptr), "cf_offload")

    def offload_static(self, cache, req_id, n_ctx, host_ptr):
        """cf_offload without any allocation: device scratch is the library's static array."""
        _check(lib.cf_offload_static(self.handle, cache.handle, req_id, n_ctx, host_ptr), "cf_offload_static")

    def inject_failure(self, nth_check):
        """Test hook: the nth post-enqueue status check of the next restore_batch fails."""
        _check(lib.cf_ctx_inject_failure(self.handle, int(nth_check)), "cf_ctx_inject_failure")

    def measure_h2d(self, host_ptr, dev_ptr, n_bytes, reps=5):
        out = C.c_double()
        _check(lib.cf_measure_h2d(self.handle, host_ptr, dev_ptr, n_bytes, reps, C.byref(out)),
               "cf_measure_h2d")
        return out.value

    def calibrate(self, cache, host_ptr, host_bytes):
        cm = cf_cost_model()
        _check(lib.cf_calibrate(self.handle, cache.handle, host_ptr, host_bytes, C.byref(cm)),
               "cf_calibrate")
        return cm

    def calibrate_overlap(self, cache, host_ptr, host_bytes, cost):
        ov = cf_overlap_model()
        _check(lib.cf_calibrate_overlap(self.handle, cache.handle, host_ptr, host_bytes, C.byref(cost),
                                        C.byref(ov)), "cf_calibrate_overlap")
        return ov

    def profile(self, kernel_names):
        mask = 0
        for n in kernel_names:
            mask |= 1 << KERNEL_NAMES.index(n)
        _check(lib.cf_ctx_profile(self.handle, mask), "cf_ctx_profile")

    def profile_read(self, reset=True):
        arr = (cf_kernel_stat * CF_N_KERNELS)()
        _check(lib.cf_ctx_profile_read(self.handle, arr, int(reset)), "cf_ctx_profile_read")
        return {KERNEL_NAMES[i]: dict(launches=arr[i].launches, total_ms=arr[i].total_ms,
                                      work=arr[i].work) for i in range(CF_N_KERNELS)}

    def read_final_hidden(self, b):
        out = np.zeros((b, self.desc.d_model), dtype=np.float32)
        _check(lib.cf_read_final_hidden(self.handle, b, out.ctypes.data), "cf_read_final_hidden")
        return out

    def op_gemm(self, A, W, W2, Cf, Dt, M, N, K, epi, impl=0, reps=1):
        ms = C.c_float()
        _check(lib.cf_op_gemm(self.handle, A, W, W2 or None, Cf or None, Dt or None, M, N, K, epi,
                              impl, reps, C.byref(ms)), "cf_op_gemm")
        return ms.value
