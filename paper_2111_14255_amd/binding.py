"""Thin ctypes binding of libmtsched.so: same names as include/mtsched.h, argument marshalling only.

The library is loaded from this directory.  There is no fallback: if it has not been built
(python -m paper_2111_14255_amd.build) loading raises.
"""
import ctypes as C
import os

from . import build as _build

MT_MAX_TENANTS = 16
MT_MAX_STAGES = 16
MT_STATIC_SCRATCH_BYTES = 16 << 20

MT_OK = 0
MT_ERR_INVALID_ARG = -1
MT_ERR_INVALID_SCHEDULE = -2
MT_ERR_SHAPE_MISMATCH = -3
MT_ERR_OUT_OF_MEMORY = -4
MT_ERR_HIP = -5
MT_ERR_NOT_FINALIZED = -6

MT_F32, MT_F16, MT_BF16 = 0, 1, 2
MT_CONV, MT_DWCONV, MT_MAXPOOL, MT_AVGPOOL, MT_GLOBAL_AVGPOOL, MT_FC, MT_LRN, MT_ADD = range(8)
MT_ACT_NONE, MT_ACT_RELU, MT_ACT_RELU6 = 0, 1, 2
MT_ISSUE_BFS, MT_ISSUE_DFS = 0, 1
MT_SCHED_GRAPH = 1
MT_SCHED_PARALLEL_ISSUE = 2
MT_SCHED_TIME_FIRST_OP = 4
MT_SCHED_SHARE_PER_STAGE = 8
MT_SCHED_FUSE_DEPTHWISE = 16
MT_SCHED_FUSE_EXPAND = 64
MT_SCHED_FUSE_POOL = 128
MT_SCHED_PRIORITIZE_SHORT = 256
MT_SCHED_TIME_TENANTS = 512
MT_SCHED_HOST_BARRIER = 1024
MT_SCHED_STREAM_GRAPHS = 32
MT_SCHED_COUNTER_BARRIER = 2048
MT_SCHED_COISSUE = 4096
MT_SEARCH_COORDINATE, MT_SEARCH_RANDOM = 0, 1


class mt_op_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "kind", "in_tensor", "res_tensor", "out_tensor", "out_c", "out_c_offset", "out_c_total",
        "r", "s", "stride_h", "stride_w", "pad_h", "pad_w", "act", "groups")] + [
        ("lrn_alpha", C.c_float), ("lrn_beta", C.c_float), ("lrn_k", C.c_float)]


class mt_op_info(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "kind", "in_h", "in_w", "in_c", "out_h", "out_w", "out_c", "kernel_id", "split_k", "grid_blocks")] + [
        ("flops", C.c_double), ("bytes", C.c_double)]


class mt_device_info(C.Structure):
    _fields_ = [("cu_count", C.c_int32), ("wavefront_size", C.c_int32), ("lds_bytes_per_block", C.c_int32),
                ("clock_khz", C.c_int32), ("l2_bytes", C.c_int64), ("hbm_bytes", C.c_int64),
                ("name", C.c_char * 64), ("arch", C.c_char * 64)]


class mt_timings(C.Structure):
    _fields_ = [("makespan_ms", C.c_float), ("host_issue_ms", C.c_float), ("n_launches", C.c_int32),
                ("n_stages", C.c_int32), ("stage_ms", C.c_float * MT_MAX_STAGES),
                ("first_op_done_ms", C.c_float * MT_MAX_TENANTS), ("n_fused", C.c_int32),
                ("tenant_done_ms", C.c_float * MT_MAX_TENANTS)]


class mt_search_opts(C.Structure):
    _fields_ = [("algo", C.c_int32), ("n_stages", C.c_int32), ("rounds", C.c_int32), ("candidates", C.c_int32),
                ("runs", C.c_int32), ("warmup", C.c_int32), ("issue_order", C.c_int32), ("flags", C.c_int32),
                ("seed_baselines", C.c_int32), ("cu_share_rounds", C.c_int32), ("wave_priority_rounds", C.c_int32),
                ("search_concurrency", C.c_int32), ("playoff_top", C.c_int32), ("playoff_runs", C.c_int32),
                ("seed", C.c_uint64)]


mt_cost_fn = C.CFUNCTYPE(C.c_double, C.POINTER(C.c_int32), C.c_void_p)
mt_share_cost_fn = C.CFUNCTYPE(C.c_double, C.POINTER(C.c_int32), C.c_void_p)

_vp, _i32, _i64, _sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
_pi32, _pf, _pd = C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_double)

# name -> (restype, argtypes); every function include/mtsched.h declares
SIGNATURES = {
    "mt_last_error": (C.c_char_p, []),
    "mt_kernel_name": (C.c_char_p, [_i32]),
    "mt_create": (_i32, [_i32, C.POINTER(_vp)]),
    "mt_destroy": (_i32, [_vp]),
    "mt_get_device_info": (_i32, [_vp, C.POINTER(mt_device_info)]),
    "mt_probe_dispatch_latency": (_i32, [_vp, _i32, _i32, _i32, _pf]),
    "mt_probe_stream_conflicts": (_i32, [_vp, _i32, _i32, _pf, _pf]),
    "mt_probe_barrier_cost": (_i32, [_vp, _i32, _i32, _i32, _pf]),
    "mt_probe_cu_mask": (_i32, [_vp, _i32, _i32, _i32, C.POINTER(C.c_uint32)]),
    "mt_probe_peak_mfma": (_i32, [_vp, _i32, _i32, _pf]),
    "mt_probe_peak_stream": (_i32, [_vp, _i32, C.c_size_t, _i32, _i32, _pf]),
    "mt_model_begin": (_i32, [_i32, _i32, _i32, _i32, _i32, C.POINTER(_vp)]),
    "mt_model_add_op": (_i32, [_vp, C.POINTER(mt_op_desc), _pi32]),
    "mt_model_end": (_i32, [_vp]),
    "mt_model_destroy": (_i32, [_vp]),
    "mt_model_num_ops": (_i32, [_vp, _pi32]),
    "mt_model_op_info": (_i32, [_vp, _i32, C.POINTER(mt_op_info)]),
    "mt_model_out_features": (_i32, [_vp, C.POINTER(_i64)]),
    "mt_model_set_weights": (_i32, [_vp, _i32, _vp, _sz, _pf, _sz]),
    "mt_model_arena_bytes": (_i32, [_vp, C.POINTER(_sz)]),
    "mt_fold_bn": (_i32, [_pf, _i64, _i64, _pf, _pf, _pf, _pf, C.c_float, _pf]),
    "mt_round_to_storage": (_i32, [_pf, _i64, _i32, _vp]),
    "mt_register": (_i32, [_vp, _vp, _vp, _sz, _pi32]),
    "mt_num_tenants": (_i32, [_vp, _pi32]),
    "mt_tenant_num_ops": (_i32, [_vp, _i32, _pi32]),
    "mt_tenant_op_info": (_i32, [_vp, _i32, _i32, C.POINTER(mt_op_info)]),
    "mt_tenant_read_tensor": (_i32, [_vp, _i32, _i32, _vp, _sz]),
    "mt_schedule_create": (_i32, [_vp, _i32, _i32, _pi32, _pi32, _pi32, _i32, _i32, C.POINTER(_vp)]),
    "mt_release_idle_streams": (_i32, [_vp]),
    "mt_schedule_set_wave_priority": (_i32, [_vp, C.POINTER(C.c_int32)]),
    "mt_schedule_destroy": (_i32, [_vp]),
    "mt_expand_pointers": (_i32, [_i32, _pi32, _i32, _pi32, _pi32]),
    "mt_issue_order_of_stage": (_i32, [_i32, _pi32, _i32, _i32, _pi32, _pi32]),
    "mt_run": (_i32, [_vp, _vp, C.POINTER(_vp), C.POINTER(_vp), C.POINTER(mt_timings)]),
    "mt_run_static_scratch": (_i32, [_vp, _vp, C.POINTER(_vp), C.POINTER(_vp), C.POINTER(mt_timings)]),
    "mt_profile_ops": (_i32, [_vp, _i32, _vp, _vp, _i32, _pf]),
    "mt_search_pointers": (_i32, [_i32, _pi32, C.POINTER(mt_search_opts), mt_cost_fn, _vp, _pi32, _pd, _pi32, _pd, _i32, _pi32]),
    "mt_playoff_pointers": (_i32, [_i32, _pi32, _i32, _pi32, _pd, _i32, _i32, mt_cost_fn, _vp, _pi32, _pd, _pi32]),
    "mt_search_cu_share": (_i32, [_i32, _i32, _i32, mt_share_cost_fn, _vp, _pi32, _pd]),
    "mt_proportional_cu_share": (_i32, [_i32, _i32, _pd, _pi32]),
    "mt_search": (_i32, [_vp, C.POINTER(mt_search_opts), C.POINTER(_vp), C.POINTER(_vp), _pi32, _pi32, _pi32, _pi32, _pd, _pi32, _pd, _i32, _pi32]),
    "mt_search_wave_priority": (_i32, [_i32, _i32, mt_share_cost_fn, _vp, _pi32, _pd]),
}

_lib = None


def load():
    """Loads the built library (building it first only if it has never been built)."""
    global _lib
    if _lib is None:
        path = os.environ.get("MTSCHED_LIB") or _build.lib_path()   # override: load another build of the library
        if not os.path.exists(path):
            _build.build()
        lib = C.CDLL(path)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


class MtError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("mtsched error %d: %s" % (code, msg))
        self.code = code


def check(code):
    if code != MT_OK:
        raise MtError(code, load().mt_last_error().decode())
    return code


def __getattr__(name):
    if name in SIGNATURES:
        return getattr(load(), name)
    raise AttributeError(name)
