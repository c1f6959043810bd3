"""ctypes binding of libss.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/ss.h)
and does nothing but convert NumPy arrays / integers to pointers and sizes and
turn a negative return code into SsError.  All work happens in the library.
There is no fallback: if the library is missing, import fails loudly.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libss.so")

if not os.path.exists(LIB_PATH):
    raise ImportError("libss.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(or python paper_2509_11076_amd/build.py) first; there is no CPU fallback")
# PyTorch ships its own HIP runtime.  libss must bind to that same copy (one runtime per
# process: streams and device pointers are shared with torch), so torch is loaded first.
import torch  # noqa: E402,F401
_lib = C.CDLL(LIB_PATH)

# ---- record layouts (mirror include/ss.h) ------------------------------------
OP_DT = np.dtype([("op_token", "<u4"), ("stack_hash", "<u4"), ("sig", "<u4"), ("n_out", "<u4")])
EVENT_DT = np.dtype([("op_idx", "<u4"), ("tensor_id", "<u4"), ("delta", "<i8")])
TENSOR_DT = np.dtype([("tensor_id", "<u4"), ("dtype", "<u4"), ("producer_op", "<u4"), ("out_slot", "<u4"),
                      ("alloc_op", "<u4"), ("last_fwd_use", "<u4"), ("first_bwd_use", "<u4"),
                      ("free_op", "<u4"), ("dev_off", "<u8"), ("dev_off_in", "<u8"), ("nbytes", "<u8")])
ANCHOR_DT = np.dtype([("ref_op", "<u4"), ("out_slot", "<u4")])
POLICY_DT = np.dtype([("ref_op", "<u4"), ("out_slot", "<u4"), ("tensor_id", "<u4"), ("flags", "<u4"),
                      ("t_out", "<u4"), ("t_free", "<u4"), ("t_in", "<u4"), ("t_use", "<u4"),
                      ("nbytes", "<u8")])
DESC_DT = np.dtype([("dev_off", "<u8"), ("host_off", "<u8"), ("nbytes", "<u8"),
                    ("tensor_id", "<u4"), ("flags", "<u4")])
ACTION_DT = np.dtype([("op_idx", "<u4"), ("kind", "<u4"), ("tensor_id", "<u4"), ("batch", "<u4")])

SS_OK = 0
SS_E_INVAL, SS_E_NOMEM, SS_E_HIP, SS_E_INFEASIBLE, SS_E_ORDER, SS_E_STATE, SS_E_CAPACITY = -1, -2, -3, -4, -6, -8, -9
SS_E_TIMEOUT = -10
SS_ACT_IN, SS_ACT_WAIT_IN, SS_ACT_OUT, SS_ACT_FREE = 0, 1, 2, 3
SS_PATH_AUTO, SS_PATH_KERNEL, SS_PATH_ENGINE, SS_PATH_STAGED = 0, 1, 2, 3
SS_CFG_TIMING, SS_CFG_POISON_FREE, SS_CFG_KEEP_LATE, SS_CFG_SYSTEM_FENCE, SS_CFG_POLICY_POINTS = 1, 2, 4, 8, 16
SS_CFG_STALL_TIMING = 32
SS_CFG_BARE_RING = 64
SS_CFG_MEMORY_MARKERS = 128
SS_SYNC_FREE, SS_SYNC_WAIT_IN, SS_SYNC_DRAIN, SS_SYNC_ITERATION_END = 0, 1, 2, 3
SS_MATCH_STEP_STAGE, SS_MATCH_HISTOGRAM, SS_MATCH_ALIGN = 1, 2, 4
SS_LEVEL_ALIGN = 3
SS_STAGE_WARMUP, SS_STAGE_GENPOLICY, SS_STAGE_STABLE = 0, 1, 2
SS_F_UNMATCHED, SS_F_ORDER, SS_F_LATE, SS_F_RESIZED, SS_F_FORCED = 1, 2, 4, 8, 16
SS_NONE_OP = 0xFFFFFFFF


class ss_config_t(C.Structure):
    _fields_ = [("staging_bytes", C.c_uint64), ("link_bytes_per_op", C.c_uint64),
                ("prefetch_bytes_per_op", C.c_uint64), ("engine_min_bytes", C.c_uint64), ("align", C.c_uint32), ("guard_bytes", C.c_uint32),
                ("stage_m", C.c_uint32), ("stage_n", C.c_uint32), ("copy_path", C.c_uint32),
                ("copy_path_in", C.c_uint32),
                ("copy_workgroups", C.c_uint32), ("copy_workgroups_out", C.c_uint32),
                ("copy_unroll", C.c_uint32), ("max_ops", C.c_uint32), ("max_events", C.c_uint32),
                ("flags", C.c_uint32), ("engine_min_bytes_out", C.c_uint64),
                ("out_streams", C.c_uint32), ("in_streams", C.c_uint32),
                ("ring_bytes", C.c_uint64), ("ring_slot_bytes", C.c_uint64),
                ("gather_workgroups", C.c_uint32), ("ring_taper", C.c_uint32),
                ("copy_desc_lookup", C.c_uint32), ("copy_cus", C.c_uint32),
                ("engine_window_in", C.c_uint32), ("engine_window_out", C.c_uint32),
                ("flag_wait_ms", C.c_uint32), ("reserved0", C.c_uint32)]


class ss_scan_result_t(C.Structure):
    _fields_ = [("peak", C.c_int64), ("final_total", C.c_int64), ("argpeak_op", C.c_int32),
                ("n_over", C.c_uint32), ("sorted", C.c_uint32), ("reserved", C.c_uint32)]


class ss_match_result_t(C.Structure):
    _fields_ = [("dot", C.c_uint64), ("na", C.c_uint64), ("nb", C.c_uint64), ("similar", C.c_uint32),
                ("stage", C.c_uint32), ("stable_step", C.c_uint32), ("n_unmatched", C.c_uint32)]


class ss_apply_result_t(C.Structure):
    _fields_ = [("staging_bytes", C.c_uint64), ("bytes_out", C.c_uint64), ("n_kept", C.c_uint32),
                ("n_dropped", C.c_uint32), ("n_late", C.c_uint32), ("n_out_batches", C.c_uint32),
                ("n_in_batches", C.c_uint32), ("reserved", C.c_uint32)]


class ss_align_result_t(C.Structure):
    _fields_ = [("lcs", C.c_uint32), ("distance", C.c_uint32), ("n_keys", C.c_uint32), ("n_unmatched", C.c_uint32)]


class ss_gen_params_t(C.Structure):
    _fields_ = [("g_fwd", C.c_uint32), ("g_bwd", C.c_uint32), ("c_num", C.c_uint32), ("c_den", C.c_uint32),
                ("min_bytes", C.c_uint64), ("phase_bytes_per_op", C.c_uint64 * 3)]


class ss_gen_result_t(C.Structure):
    _fields_ = [("peak_no_swap", C.c_int64), ("peak_with_policy", C.c_int64),
                ("n_over_with_policy", C.c_uint32), ("n_rounds", C.c_uint32), ("n_items", C.c_uint32),
                ("n_late", C.c_uint32), ("bytes", C.c_uint64)]


class ss_stats_t(C.Structure):
    _fields_ = [("bytes_out", C.c_uint64), ("bytes_in", C.c_uint64), ("kernel_batches", C.c_uint64),
                ("engine_batches", C.c_uint64), ("free_waits", C.c_uint64), ("in_waits", C.c_uint64),
                ("ops_recorded", C.c_uint64), ("events_recorded", C.c_uint64),
                ("last_hip_error", C.c_int32), ("engine_batches_out", C.c_uint32),
                ("match_levels", C.c_uint64 * 5), ("reuse_hist", C.c_uint32 * 16),
                ("reuse_sum", C.c_uint64), ("reuse_count", C.c_uint64),
                ("stall_free_ms", C.c_double), ("stall_wait_in_ms", C.c_double),
                ("ring_batches", C.c_uint64), ("ring_transfers", C.c_uint64),
                ("ring_batches_in", C.c_uint64), ("ring_transfers_in", C.c_uint64),
                ("engine_window_waits", C.c_uint64)]


class ss_bw_t(C.Structure):
    _fields_ = [("d2h_gbps", C.c_double), ("h2d_gbps", C.c_double), ("bidir_d2h_gbps", C.c_double),
                ("bidir_h2d_gbps", C.c_double), ("kernel_d2h_gbps", C.c_double),
                ("kernel_h2d_gbps", C.c_double), ("kernel_bidir_d2h_gbps", C.c_double),
                ("kernel_bidir_h2d_gbps", C.c_double)]


class SsError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = "%s: %s (%d)" % (where, ss_strerror(code), code)
        if code in (SS_E_HIP, SS_E_NOMEM):
            msg += " [last HIP error: %s]" % (ss_last_hip_error(),)
        super().__init__(msg)


_P = C.c_void_p
_lib.ss_strerror.restype = C.c_char_p
_lib.ss_strerror.argtypes = [C.c_int]
_SIGS = {
    "ss_config_default": [C.POINTER(ss_config_t)],
    "ss_create": [C.POINTER(_P), C.POINTER(ss_config_t)],
    "ss_destroy": [_P],
    "ss_bind": [_P, _P, C.c_uint64, _P],
    "ss_intern_op": [_P, C.c_char_p, C.c_char_p, C.c_uint32, C.c_uint32, C.c_uint32, _P],
    "ss_trace_begin": [_P],
    "ss_trace_record": [_P, _P, _P, C.c_uint32],
    "ss_trace_view": [_P, C.POINTER(_P), C.POINTER(C.c_uint32), C.POINTER(_P), C.POINTER(C.c_uint64),
                      C.POINTER(C.c_int64)],
    "ss_timeline_scan": [_P, _P, C.c_uint64, _P, C.c_uint64, C.c_uint32, C.c_int64, C.c_int64, _P, _P, _P,
                         C.POINTER(ss_scan_result_t)],
    "ss_match_sequence": [_P, _P, C.c_uint32, _P, C.c_uint32, _P, C.c_uint32, C.c_uint32, _P, _P,
                          C.POINTER(ss_match_result_t)],
    "ss_apply_policy": [_P, _P, C.c_uint32, _P, _P, C.c_uint32, _P, _P, C.POINTER(C.c_uint32), _P, _P, _P,
                        C.POINTER(C.c_uint32), C.POINTER(ss_apply_result_t)],
    "ss_schedule_view": [_P, C.POINTER(_P), C.POINTER(C.c_uint32), C.POINTER(_P), C.POINTER(C.c_uint32),
                         C.POINTER(_P)],
    "ss_load_schedule": [_P, _P, C.c_uint32, _P, C.c_uint32, _P, C.c_uint32, _P, C.c_uint32, _P],
    "ss_greedy_policy": [_P, _P, C.c_uint32, _P, C.c_uint64, C.c_uint32, C.c_int64, C.c_int64, C.c_uint64,
                         _P, C.c_uint32, _P, C.POINTER(C.c_uint32), C.POINTER(C.c_int64)],
    "ss_timeline_scan_batch": [_P, _P, C.c_uint64, _P, _P, C.c_uint32, C.c_uint32, C.c_int64, C.c_int64, _P, _P],
    "ss_timeline_scan_static": [_P, _P, _P, C.c_uint64, _P, C.c_uint64, C.c_uint32, C.c_int64, C.c_int64, _P, _P, _P, _P],
    "ss_batch_done": [_P, C.c_uint32, C.c_uint32, C.POINTER(C.c_int)],
    "ss_trace_event": [_P, C.c_uint32, C.c_int64],
    "ss_trace_amend": [_P, C.c_uint32, C.c_uint32, C.c_uint32],
    "ss_align_sequence": [_P, _P, C.c_uint32, _P, C.c_uint32, _P, C.c_uint32, _P, _P, _P,
                          C.POINTER(ss_align_result_t)],
    "ss_generate_policy": [_P, _P, C.c_uint32, _P, C.c_uint32, _P, C.c_uint64, C.c_int64, C.c_int64,
                           C.POINTER(ss_gen_params_t), _P, C.POINTER(C.c_uint32), C.POINTER(ss_gen_result_t)],
    "ss_generate_policy_best": [_P, _P, C.c_uint32, _P, C.c_uint32, _P, C.c_uint64, C.c_int64, C.c_int64,
                                _P, C.c_uint32, _P, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32),
                                C.POINTER(ss_gen_result_t)],
    "ss_swap_out": [_P, C.c_uint32],
    "ss_swap_in": [_P, C.c_uint32],
    "ss_sync": [_P, C.c_uint32, C.c_uint32],
    "ss_dispatch": [_P, C.c_uint32, C.c_uint32],
    "ss_swap_out_from": [_P, C.c_uint32, _P],
    "ss_swap_in_to": [_P, C.c_uint32, _P],
    "ss_host_peek": [_P, C.c_uint64, C.c_uint64, C.POINTER(_P)],
    "ss_staging_fill": [_P, C.c_int],
    "ss_batch_ms": [_P, C.c_uint32, C.c_uint32, C.POINTER(C.c_float), C.POINTER(C.c_float)],
    "ss_batch_ms_all": [_P, C.c_uint32, _P, C.c_uint32, C.POINTER(C.c_uint32)],
    "ss_batch_window": [_P, C.c_uint32, C.c_uint32, C.POINTER(C.c_float), C.POINTER(C.c_float)],
    "ss_bw_probe": [_P, C.c_uint64, C.c_uint32, C.POINTER(ss_bw_t)],
    "ss_ring_view": [_P, C.c_uint32, C.POINTER(C.c_uint32), C.POINTER(_P), C.POINTER(_P)],
    "ss_get_stats": [_P, C.POINTER(ss_stats_t)],
}
for _name, _args in _SIGS.items():
    _f = getattr(_lib, _name)          # AttributeError here = the library lacks a declared symbol
    _f.argtypes = _args
    _f.restype = C.c_int
_lib.ss_last_hip_error.restype = C.c_int
_lib.ss_last_hip_error.argtypes = [C.POINTER(C.c_char_p), C.POINTER(C.c_char_p), C.POINTER(C.c_int)]
EXPORTS = sorted(list(_SIGS) + ["ss_strerror", "ss_last_hip_error"])


def ss_strerror(code):
    return _lib.ss_strerror(int(code)).decode()


def ss_last_hip_error():
    """(hipError_t, name, source file, line) of the calling thread's last failing HIP call"""
    name, file, line = C.c_char_p(), C.c_char_p(), C.c_int()
    code = _lib.ss_last_hip_error(C.byref(name), C.byref(file), C.byref(line))
    return code, (name.value or b"").decode(), os.path.basename((file.value or b"").decode()), line.value


def _ck(rc, where):
    if rc != SS_OK:
        raise SsError(rc, where)


def _arr(a, dt):
    """contiguous array of the given record type (no copy if already so); None stays None"""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype != dt:
        if a.dtype.itemsize != np.dtype(dt).itemsize or a.dtype.names != np.dtype(dt).names:
            a = a.astype(dt)
        else:
            a = a.view(dt)
    return a


def _ptr(a):
    return None if a is None or a.size == 0 else a.ctypes.data_as(_P)


def ss_config_default():
    cfg = ss_config_t()
    _ck(_lib.ss_config_default(C.byref(cfg)), "ss_config_default")
    return cfg


def ss_create(cfg=None):
    ctx = _P()
    _ck(_lib.ss_create(C.byref(ctx), C.byref(cfg) if cfg is not None else None), "ss_create")
    return ctx


def ss_destroy(ctx):
    _ck(_lib.ss_destroy(ctx), "ss_destroy")


def ss_bind(ctx, arena_ptr, arena_bytes, compute_stream):
    _ck(_lib.ss_bind(ctx, _P(int(arena_ptr or 0)), int(arena_bytes), _P(int(compute_stream or 0))), "ss_bind")


def ss_intern_op(ctx, name, stack, dtype, n_out, phase):
    op = np.zeros(1, dtype=OP_DT)
    _ck(_lib.ss_intern_op(ctx, name.encode(), stack.encode(), int(dtype), int(n_out), int(phase), _ptr(op)),
        "ss_intern_op")
    return op[0]


def ss_trace_begin(ctx):
    _ck(_lib.ss_trace_begin(ctx), "ss_trace_begin")


def ss_trace_record(ctx, op, events=None):
    op = _arr(np.asarray(op).reshape(1), OP_DT)
    ev = _arr(events, EVENT_DT)
    _ck(_lib.ss_trace_record(ctx, _ptr(op), _ptr(ev), 0 if ev is None else len(ev)), "ss_trace_record")


def ss_trace_record_prepared(ctx, ops, events):
    """Marshal a whole trace once: returns a list of zero-argument callables, one per operator,
    each of which is exactly one ss_trace_record call (for dispatch loops that must not pay
    NumPy slicing per operator).  `events` must be in operator order."""
    ops = _arr(ops, OP_DT)
    ev = _arr(events, EVENT_DT)
    bounds = np.searchsorted(ev["op_idx"], np.arange(len(ops) + 1))
    f = _lib.ss_trace_record
    op0, ev0 = ops.ctypes.data, ev.ctypes.data if len(ev) else 0
    calls = []
    for i in range(len(ops)):
        n = int(bounds[i + 1] - bounds[i])
        calls.append((_P(op0 + 16 * i), _P(ev0 + 16 * int(bounds[i])) if n else None, n))
    keep = (ops, ev)           # the arrays must outlive the pointers

    def record(i, _f=f, _c=calls, _ctx=ctx, _keep=keep):
        rc = _f(_ctx, *_c[i])
        if rc != SS_OK:
            raise SsError(rc, "ss_trace_record")
    return record


def ss_batch_done(ctx, direction, batch):
    d = C.c_int(0)
    _ck(_lib.ss_batch_done(ctx, int(direction), int(batch), C.byref(d)), "ss_batch_done")
    return bool(d.value)


def ss_trace_event(ctx, tensor_id, delta):
    _ck(_lib.ss_trace_event(ctx, int(tensor_id), int(delta)), "ss_trace_event")


def ss_trace_amend(ctx, op_idx, dtype, n_out):
    _ck(_lib.ss_trace_amend(ctx, int(op_idx), int(dtype), int(n_out)), "ss_trace_amend")


def ss_trace_view(ctx):
    """(ops, events, balance) as NumPy copies of the library's pinned arrays"""
    po, pe = _P(), _P()
    n, ne, bal = C.c_uint32(), C.c_uint64(), C.c_int64()
    _ck(_lib.ss_trace_view(ctx, C.byref(po), C.byref(n), C.byref(pe), C.byref(ne), C.byref(bal)), "ss_trace_view")
    ops = np.frombuffer((C.c_char * (n.value * OP_DT.itemsize)).from_address(po.value), dtype=OP_DT).copy() \
        if n.value else np.zeros(0, OP_DT)
    ev = np.frombuffer((C.c_char * (ne.value * EVENT_DT.itemsize)).from_address(pe.value), dtype=EVENT_DT).copy() \
        if ne.value else np.zeros(0, EVENT_DT)
    return ops, ev, bal.value


def ss_timeline_scan(ctx, events, policy_events, n_ops, base, budget, want_timeline=False, want_per_op=True):
    ev = _arr(events, EVENT_DT)
    pe = _arr(policy_events, EVENT_DT)
    n_ev = 0 if ev is None else len(ev)
    n_pe = 0 if pe is None else len(pe)
    tl = np.zeros(n_ev + n_pe, dtype=np.int64) if want_timeline else None
    per_op = np.zeros(n_ops, dtype=np.int64) if want_per_op else None
    mre = np.zeros(n_ops, dtype=np.int64) if want_per_op else None
    res = ss_scan_result_t()
    # an empty output array still needs a non-null pointer to be "wanted"
    tlp = None if tl is None else tl.ctypes.data_as(_P)
    _ck(_lib.ss_timeline_scan(ctx, _ptr(ev), n_ev, _ptr(pe), n_pe, int(n_ops), int(base), int(budget),
                              tlp, _ptr(per_op), _ptr(mre), C.byref(res)), "ss_timeline_scan")
    return dict(timeline=tl, per_op=per_op, mre=mre, peak=res.peak, argpeak_op=res.argpeak_op,
                n_over=res.n_over, final=res.final_total, sorted=res.sorted)


def ss_timeline_scan_static(ctx, stream, d_ev, n_ev, d_pev, n_pe, n_ops, base, budget, d_timeline, d_per_op, d_mre,
                            d_res):
    """every d_* is a device address (int, 0 = NULL); only enqueues: synchronise the stream before reading"""
    def p(x):
        return _P(int(x)) if x else None
    _ck(_lib.ss_timeline_scan_static(ctx, p(stream), p(d_ev), int(n_ev), p(d_pev), int(n_pe), int(n_ops), int(base),
                                     int(budget), p(d_timeline), p(d_per_op), p(d_mre), p(d_res)),
        "ss_timeline_scan_static")


def ss_timeline_scan_batch(ctx, events, policy_event_lists, n_ops, base, budget, want_per_op=False):
    """policy_event_lists: one EVENT_DT array (or None) per candidate; returns a list of result dicts"""
    ev = _arr(events, EVENT_DT)
    lists = [np.zeros(0, EVENT_DT) if p is None else _arr(p, EVENT_DT) for p in policy_event_lists]
    k = len(lists)
    start = np.zeros(k + 1, dtype=np.uint64)
    start[1:] = np.cumsum([len(p) for p in lists])
    pev = np.concatenate(lists) if k and int(start[-1]) else np.zeros(0, EVENT_DT)
    res = (ss_scan_result_t * max(1, k))()
    per_op = np.zeros((k, n_ops), dtype=np.int64) if want_per_op else None
    pp = None if per_op is None or per_op.size == 0 else per_op.ctypes.data_as(_P)
    _ck(_lib.ss_timeline_scan_batch(ctx, _ptr(ev), 0 if ev is None else len(ev), _ptr(pev), _ptr(start), k, int(n_ops),
                                    int(base), int(budget), pp, C.cast(res, _P)), "ss_timeline_scan_batch")
    out = []
    for c in range(k):
        r = res[c]
        out.append(dict(peak=r.peak, final=r.final_total, argpeak_op=r.argpeak_op, n_over=r.n_over,
                        per_op=None if per_op is None else per_op[c]))
    return out


def ss_match_sequence(ctx, ref, cur, anchors, flags=0):
    ref = _arr(ref, OP_DT)
    cur = _arr(cur, OP_DT)
    anc = _arr(anchors, ANCHOR_DT)
    k = 0 if anc is None else len(anc)
    new_idx = np.full(k, -1, dtype=np.int32)
    level = np.full(k, 255, dtype=np.uint8)
    res = ss_match_result_t()
    _ck(_lib.ss_match_sequence(ctx, _ptr(ref), len(ref), _ptr(cur), len(cur), _ptr(anc), k, int(flags),
                               _ptr(new_idx), _ptr(level), C.byref(res)), "ss_match_sequence")
    return dict(similar=bool(res.similar), dot=res.dot, na=res.na, nb=res.nb, stage=res.stage,
                stable_step=res.stable_step, new_idx=new_idx, level=level, n_unmatched=res.n_unmatched)


def ss_align_sequence(ctx, ref, cur, anchors=None):
    ref = _arr(ref, OP_DT)
    cur = _arr(cur, OP_DT)
    anc = _arr(anchors, ANCHOR_DT)
    k = 0 if anc is None else len(anc)
    n = 0 if ref is None else len(ref)
    m = 0 if cur is None else len(cur)
    ref_to_cur = np.full(n, -2, dtype=np.int32)
    new_idx = np.full(k, -1, dtype=np.int32)
    level = np.full(k, 255, dtype=np.uint8)
    res = ss_align_result_t()
    _ck(_lib.ss_align_sequence(ctx, _ptr(ref), n, _ptr(cur), m, _ptr(anc), k, _ptr(ref_to_cur), _ptr(new_idx),
                               _ptr(level), C.byref(res)), "ss_align_sequence")
    return dict(ref_to_cur=ref_to_cur, new_idx=new_idx, level=level, lcs=res.lcs, distance=res.distance,
                n_keys=res.n_keys, n_unmatched=res.n_unmatched)


def ss_apply_policy(ctx, policy, new_idx, tensors, allow_nomem=False):
    """allow_nomem: a schedule that needs more staging than the context owns is still returned
    (the library fills every output before it reports SS_E_NOMEM); it is then not loaded."""
    pol = _arr(policy, POLICY_DT)
    idx = np.ascontiguousarray(new_idx, dtype=np.int32)
    tab = _arr(tensors, TENSOR_DT)
    k = len(pol)
    resolved = np.zeros(k, dtype=POLICY_DT)
    actions = np.zeros(4 * k, dtype=ACTION_DT)
    d_out = np.zeros(k, dtype=DESC_DT)
    d_in = np.zeros(k, dtype=DESC_DT)
    pev = np.zeros(2 * k, dtype=EVENT_DT)
    na, npe = C.c_uint32(4 * k), C.c_uint32(2 * k)
    res = ss_apply_result_t()
    rc = _lib.ss_apply_policy(ctx, _ptr(pol), k, _ptr(idx), _ptr(tab), len(tab), _ptr(resolved), _ptr(actions),
                              C.byref(na), _ptr(d_out), _ptr(d_in), _ptr(pev), C.byref(npe), C.byref(res))
    if not (allow_nomem and rc == SS_E_NOMEM):
        _ck(rc, "ss_apply_policy")
    kept = res.n_kept
    out = dict(resolved=resolved, actions=actions[:na.value], descs_out=d_out[:kept], descs_in=d_in[:kept],
               policy_events=pev[:npe.value], staging_bytes=res.staging_bytes, bytes_out=res.bytes_out,
               n_kept=kept, n_dropped=res.n_dropped, n_late=res.n_late,
               n_out_batches=res.n_out_batches, n_in_batches=res.n_in_batches, rc=rc)
    return out


def ss_schedule_view(ctx):
    po, pi, pd = _P(), _P(), _P()
    no, ni = C.c_uint32(), C.c_uint32()
    _ck(_lib.ss_schedule_view(ctx, C.byref(po), C.byref(no), C.byref(pi), C.byref(ni), C.byref(pd)),
        "ss_schedule_view")

    def grab(p, n):
        return np.frombuffer((C.c_char * (4 * n)).from_address(p.value), dtype=np.uint32).copy() if n else \
            np.zeros(0, np.uint32)
    return grab(po, no.value + 1), grab(pi, ni.value + 1), grab(pd, ni.value)


def ss_load_schedule(ctx, descs_out, out_start, descs_in, in_start, in_dep=None):
    do, di = _arr(descs_out, DESC_DT), _arr(descs_in, DESC_DT)
    os_ = np.ascontiguousarray(out_start, dtype=np.uint32)
    is_ = np.ascontiguousarray(in_start, dtype=np.uint32)
    dep = None if in_dep is None else np.ascontiguousarray(in_dep, dtype=np.uint32)
    _ck(_lib.ss_load_schedule(ctx, _ptr(do), len(do), _ptr(os_), max(len(os_) - 1, 0), _ptr(di), len(di),
                              _ptr(is_), max(len(is_) - 1, 0), _ptr(dep)), "ss_load_schedule")


def ss_greedy_policy(ctx, tensors, events, n_ops, base, budget, min_bytes=0, initial=None):
    tab = _arr(tensors, TENSOR_DT)
    ev = _arr(events, EVENT_DT)
    ini = _arr(initial, POLICY_DT)
    out = np.zeros(len(tab) + (0 if ini is None else len(ini)), dtype=POLICY_DT)
    n = C.c_uint32(len(out))
    peak = C.c_int64()
    _ck(_lib.ss_greedy_policy(ctx, _ptr(tab), len(tab), _ptr(ev), len(ev), int(n_ops), int(base), int(budget),
                              int(min_bytes), _ptr(ini), 0 if ini is None else len(ini), _ptr(out),
                              C.byref(n), C.byref(peak)), "ss_greedy_policy")
    return out[:n.value], peak.value


def _gen_params(g_fwd, g_bwd, c_num=1, c_den=1, min_bytes=0, phase_bytes_per_op=None):
    p = ss_gen_params_t(int(g_fwd), int(g_bwd), int(c_num), int(c_den), int(min_bytes))
    for i, b in enumerate(phase_bytes_per_op or ()):
        p.phase_bytes_per_op[i] = int(b)
    return p


def ss_generate_policy(ctx, ops, tensors, events, base, limit, g_fwd, g_bwd, c_num=1, c_den=1, min_bytes=0,
                       phase_bytes_per_op=None):
    ops = _arr(ops, OP_DT)
    tab = _arr(tensors, TENSOR_DT)
    ev = _arr(events, EVENT_DT)
    prm = _gen_params(g_fwd, g_bwd, c_num, c_den, min_bytes, phase_bytes_per_op)
    out = np.zeros(len(tab), dtype=POLICY_DT)
    n = C.c_uint32(len(out))
    res = ss_gen_result_t()
    _ck(_lib.ss_generate_policy(ctx, _ptr(ops), len(ops), _ptr(tab), len(tab), _ptr(ev), len(ev), int(base),
                                int(limit), C.byref(prm), _ptr(out), C.byref(n), C.byref(res)),
        "ss_generate_policy")
    return out[:n.value], {f: getattr(res, f) for f, _ in ss_gen_result_t._fields_}


def ss_generate_policy_best(ctx, ops, tensors, events, base, limit, param_sets):
    """param_sets: list of dicts(g_fwd, g_bwd[, c_num, c_den, min_bytes]); returns (policy, result, chosen)"""
    ops = _arr(ops, OP_DT)
    tab = _arr(tensors, TENSOR_DT)
    ev = _arr(events, EVENT_DT)
    prm = (ss_gen_params_t * max(1, len(param_sets)))()
    for i, d in enumerate(param_sets):
        prm[i] = _gen_params(**d)
    out = np.zeros(len(tab), dtype=POLICY_DT)
    n, chosen = C.c_uint32(len(out)), C.c_uint32(0)
    res = ss_gen_result_t()
    _ck(_lib.ss_generate_policy_best(ctx, _ptr(ops), len(ops), _ptr(tab), len(tab), _ptr(ev), len(ev), int(base),
                                     int(limit), C.cast(prm, _P), len(param_sets), _ptr(out), C.byref(n),
                                     C.byref(chosen), C.byref(res)), "ss_generate_policy_best")
    return out[:n.value], {f: getattr(res, f) for f, _ in ss_gen_result_t._fields_}, chosen.value


def ss_swap_out(ctx, batch):
    _ck(_lib.ss_swap_out(ctx, int(batch)), "ss_swap_out")


def ss_swap_in(ctx, batch):
    _ck(_lib.ss_swap_in(ctx, int(batch)), "ss_swap_in")


def _addr_array(addrs):
    a = np.ascontiguousarray(addrs, dtype=np.uint64)
    return a, (a.ctypes.data_as(_P) if len(a) else None)


def ss_swap_out_from(ctx, batch, dev_src):
    """dev_src: one device address per tensor of the batch"""
    keep, p = _addr_array(dev_src)
    _ck(_lib.ss_swap_out_from(ctx, int(batch), p), "ss_swap_out_from")


def ss_swap_in_to(ctx, batch, dev_dst):
    """dev_dst: one device address per tensor of the batch"""
    keep, p = _addr_array(dev_dst)
    _ck(_lib.ss_swap_in_to(ctx, int(batch), p), "ss_swap_in_to")


def ss_sync(ctx, what, ident=0):
    _ck(_lib.ss_sync(ctx, int(what), int(ident)), "ss_sync")


def ss_dispatch(ctx, op_idx, when):
    """every scheduled action before (when = 0) or after (when = 1) operator op_idx"""
    _ck(_lib.ss_dispatch(ctx, int(op_idx), int(when)), "ss_dispatch")


def ss_host_peek(ctx, host_off, nbytes):
    """NumPy uint8 view (no copy) of a piece of the pinned staging area"""
    p = _P()
    _ck(_lib.ss_host_peek(ctx, int(host_off), int(nbytes), C.byref(p)), "ss_host_peek")
    if nbytes == 0:
        return np.zeros(0, np.uint8)
    return np.frombuffer((C.c_char * int(nbytes)).from_address(p.value), dtype=np.uint8)


def ss_staging_fill(ctx, byte):
    _ck(_lib.ss_staging_fill(ctx, int(byte)), "ss_staging_fill")


def ss_batch_ms(ctx, direction, batch=None):
    """(ms of one batch or None, span ms over all batches of that direction)"""
    ms, span = C.c_float(), C.c_float()
    _ck(_lib.ss_batch_ms(ctx, int(direction), 0 if batch is None else int(batch),
                         C.byref(ms) if batch is not None else None, C.byref(span)), "ss_batch_ms")
    return (ms.value if batch is not None else None), span.value


def ss_batch_ms_all(ctx, direction, capacity=65536):
    """durations (ms) of every unit of a direction in the iteration drained last; -1 where a unit did not run"""
    out = np.zeros(capacity, dtype=np.float32)
    n = C.c_uint32()
    _ck(_lib.ss_batch_ms_all(ctx, int(direction), out.ctypes.data_as(_P), capacity, C.byref(n)), "ss_batch_ms_all")
    return out[:n.value].copy()


def ss_batch_window(ctx, direction, batch):
    a, b = C.c_float(), C.c_float()
    _ck(_lib.ss_batch_window(ctx, int(direction), int(batch), C.byref(a), C.byref(b)), "ss_batch_window")
    return a.value, b.value


def ss_ring_view(ctx, direction=0):
    """(group_of int32[batches of that direction], group_bytes uint64[n_groups]) as copies"""
    n, g, gb = C.c_uint32(), _P(), _P()
    _ck(_lib.ss_ring_view(ctx, int(direction), C.byref(n), C.byref(g), C.byref(gb)), "ss_ring_view")
    nob = len(ss_schedule_view(ctx)[1 if direction else 0]) - 1
    group_of = np.frombuffer((C.c_char * (4 * nob)).from_address(g.value), dtype=np.int32).copy() if nob and g.value \
        else np.zeros(0, np.int32)
    group_bytes = np.frombuffer((C.c_char * (8 * n.value)).from_address(gb.value), dtype=np.uint64).copy() \
        if n.value else np.zeros(0, np.uint64)
    return group_of, group_bytes


def ss_bw_probe(ctx, nbytes=1 << 30, reps=10):
    out = ss_bw_t()
    _ck(_lib.ss_bw_probe(ctx, int(nbytes), int(reps), C.byref(out)), "ss_bw_probe")
    return {f: getattr(out, f) for f, _ in ss_bw_t._fields_}


def ss_get_stats(ctx):
    st = ss_stats_t()
    _ck(_lib.ss_get_stats(ctx, C.byref(st)), "ss_get_stats")
    return {f: (list(getattr(st, f)) if hasattr(getattr(st, f), "__len__") else getattr(st, f))
            for f, _ in ss_stats_t._fields_}
