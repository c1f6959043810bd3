"""Record layouts of the arrays exchanged with the swap-executor interface.

These are the *input/output formats* only (field names, widths, order).  The
HIP library declares the same layouts in its C header; the oracle reads the
fields by name.  No arithmetic lives here.
"""
import numpy as np

# one dispatched operator (Sec. 3, Lightweight mode: integer token per operator;
# Detailed mode adds call stack and data type, kept as integers)
OP_DT = np.dtype([("op_token", "<u4"), ("stack_hash", "<u4"),
                  ("sig", "<u4"), ("n_out", "<u4")])
# one alloc (+) or free (-) of the memory trace (Sec. 3, last paragraph)
EVENT_DT = np.dtype([("op_idx", "<u4"), ("tensor_id", "<u4"), ("delta", "<i8")])
# one tensor of the current iteration
TENSOR_DT = np.dtype([("tensor_id", "<u4"), ("dtype", "<u4"),
                      ("producer_op", "<u4"), ("out_slot", "<u4"),
                      ("alloc_op", "<u4"), ("last_fwd_use", "<u4"),
                      ("first_bwd_use", "<u4"), ("free_op", "<u4"),
                      ("dev_off", "<u8"), ("dev_off_in", "<u8"), ("nbytes", "<u8")])
ANCHOR_DT = np.dtype([("ref_op", "<u4"), ("out_slot", "<u4")])
# one policy item: tensor identity + swap-out point, free point, swap-in point,
# first backward use (Sec. 4.3-4.4)
POLICY_DT = np.dtype([("ref_op", "<u4"), ("out_slot", "<u4"),
                      ("tensor_id", "<u4"), ("flags", "<u4"),
                      ("t_out", "<u4"), ("t_free", "<u4"),
                      ("t_in", "<u4"), ("t_use", "<u4"), ("nbytes", "<u8")])
DESC_DT = np.dtype([("dev_off", "<u8"), ("host_off", "<u8"), ("nbytes", "<u8"),
                    ("tensor_id", "<u4"), ("flags", "<u4")])
ACTION_DT = np.dtype([("op_idx", "<u4"), ("kind", "<u4"),
                      ("tensor_id", "<u4"), ("batch", "<u4")])

assert OP_DT.itemsize == 16 and EVENT_DT.itemsize == 16
assert TENSOR_DT.itemsize == 56 and ANCHOR_DT.itemsize == 8
assert POLICY_DT.itemsize == 40 and DESC_DT.itemsize == 32
assert ACTION_DT.itemsize == 16

NONE_OP = 0xFFFFFFFF          # "no such operator" (e.g. a tensor never used in backward)

# data-type codes carried in the low byte of `sig`
DT_BF16, DT_FP32, DT_U8 = 1, 2, 3
DT_SIZE = {DT_BF16: 2, DT_FP32: 4, DT_U8: 1}
# phase codes carried in bits 16.. of `sig`
PH_FWD, PH_BWD, PH_OPT = 0, 1, 2
