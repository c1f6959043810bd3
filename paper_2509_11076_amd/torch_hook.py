"""ctypes binding of libss_torch_hook.so (include/ss_torch_hook.h): argument marshalling only."""
import ctypes as C
import os

import torch  # noqa: F401  (the hook library links the PyTorch libraries of this process)

from . import binding as B

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libss_torch_hook.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libss_torch_hook.so is not built: run `python -m paper_2509_11076_amd.build`")
_lib = C.CDLL(LIB_PATH, mode=C.RTLD_GLOBAL)

SS_HOOK_OFF, SS_HOOK_LIGHTWEIGHT, SS_HOOK_DETAILED = 0, 1, 2


class ss_hook_stats_t(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("ops", "events", "dropped_ops", "dropped_events", "foreign_frees",
                                          "errors")]


_SIGS = {"ss_hook_install": [C.c_void_p, C.c_int], "ss_hook_set_mode": [C.c_int],
         "ss_hook_set_phase": [C.c_uint32], "ss_hook_begin_iteration": [], "ss_hook_remove": [],
         "ss_hook_get_stats": [C.POINTER(ss_hook_stats_t)],
         "ss_hook_tensor_table": [C.c_void_p, C.POINTER(C.c_uint32)],
         "ss_hook_current_op": [C.POINTER(C.c_uint32)],
         "ss_hook_pause": [C.c_int],
         "ss_hook_block_of": [C.c_void_p, C.c_void_p, C.POINTER(C.c_uint64)]}
for _n, _a in _SIGS.items():
    getattr(_lib, _n).argtypes = _a
    getattr(_lib, _n).restype = C.c_int
EXPORTS = sorted(_SIGS)


def _ck(rc, what):
    if rc != 0:
        raise B.SsError(rc, what)


def ss_hook_install(ctx, mode):
    _ck(_lib.ss_hook_install(ctx, int(mode)), "ss_hook_install")


def ss_hook_set_mode(mode):
    _ck(_lib.ss_hook_set_mode(int(mode)), "ss_hook_set_mode")


def ss_hook_set_phase(phase):
    _ck(_lib.ss_hook_set_phase(int(phase)), "ss_hook_set_phase")


def ss_hook_begin_iteration():
    _ck(_lib.ss_hook_begin_iteration(), "ss_hook_begin_iteration")


def ss_hook_remove():
    _ck(_lib.ss_hook_remove(), "ss_hook_remove")


def ss_hook_tensor_table():
    import numpy as np
    n = C.c_uint32(0)
    rc = _lib.ss_hook_tensor_table(None, C.byref(n))
    if rc not in (0, B.SS_E_CAPACITY):
        _ck(rc, "ss_hook_tensor_table")
    out = np.zeros(n.value, dtype=B.TENSOR_DT)
    if n.value:
        _ck(_lib.ss_hook_tensor_table(out.ctypes.data_as(C.c_void_p), C.byref(n)), "ss_hook_tensor_table")
    return out[:n.value]


def ss_hook_current_op():
    n = C.c_uint32()
    _ck(_lib.ss_hook_current_op(C.byref(n)), "ss_hook_current_op")
    return n.value


def ss_hook_pause(on):
    _ck(_lib.ss_hook_pause(1 if on else 0), "ss_hook_pause")


def ss_hook_block_of(dev_addr):
    """(tensor-table row, block start address) of the block of this iteration holding dev_addr, or None"""
    import numpy as np
    row = np.zeros(1, dtype=B.TENSOR_DT)
    addr = C.c_uint64()
    rc = _lib.ss_hook_block_of(C.c_void_p(int(dev_addr)), row.ctypes.data_as(C.c_void_p), C.byref(addr))
    if rc == B.SS_E_INVAL:
        return None
    _ck(rc, "ss_hook_block_of")
    return row[0], addr.value


def ss_hook_get_stats():
    st = ss_hook_stats_t()
    _ck(_lib.ss_hook_get_stats(C.byref(st)), "ss_hook_get_stats")
    return {n: getattr(st, n) for n, _ in ss_hook_stats_t._fields_}
