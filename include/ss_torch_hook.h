/* Online profiler hook inside PyTorch (SmartSwap, Sec. 3: a hook at the operator dispatch point,
 * working in Lightweight or Detailed mode).  Exported by libss_torch_hook.so, which links the
 * PyTorch libraries of the running process and libss.so; plain C ABI, no torch types.
 *
 * After ss_hook_install every operator PyTorch dispatches in this process (ATen's RecordFunction,
 * scope FUNCTION: forward operators and those the autograd nodes run) is appended to `ctx`'s trace
 * with ss_trace_record, in dispatch order:
 *   SS_HOOK_LIGHTWEIGHT  the token of the operator's name and the current phase; nothing else
 *   SS_HOOK_DETAILED     also a 32-bit hash of the innermost 8 Python frames (0 on threads the
 *                        interpreter does not know, i.e. the autograd engine's), the data-type code and
 *                        the number of tensor outputs (set when the operator returns, ss_trace_amend),
 *                        and the caching allocator's alloc / completed-free calls as events of the
 *                        operator running at that moment (ss_trace_event; the sizes asked for,
 *                        before the allocator rounds them; ids counted from 0 per iteration)
 * Data-type codes: 1 bf16, 2 fp32, 3 u8, 4 fp16, 5 i64, 6 i32, 7 bool, 8 fp64, 15 other, 0 no tensor.
 * One context at a time; calls are serialised by a lock.  The context must outlive the hook:
 * call ss_hook_remove before ss_destroy. */
#ifndef SS_TORCH_HOOK_H
#define SS_TORCH_HOOK_H
#include <stdint.h>

#include "ss.h"

#ifdef __cplusplus
extern "C" {
#endif

enum { SS_HOOK_OFF = 0, SS_HOOK_LIGHTWEIGHT = 1, SS_HOOK_DETAILED = 2 };

typedef struct {
  uint64_t ops, events;                  /* recorded since the library was loaded            */
  uint64_t dropped_ops, dropped_events;  /* refused by ss_trace_record / ss_trace_event (capacity) */
  uint64_t foreign_frees;                /* frees of blocks allocated before the iteration began
                                            (recorded too, under an id of their own)         */
  uint64_t errors;
} ss_hook_stats_t;

/* Register the callbacks (once per process) and direct them to ctx.  SS_E_INVAL on a bad mode;
 * SS_E_STATE (here, in ss_hook_set_mode and in ss_hook_remove) if PyTorch raised an error while
 * the callbacks were registered or removed: no exception leaves these functions. */
int ss_hook_install(ss_ctx *ctx, int mode);
/* Switch mode without touching the registration (Algo. 1: Detailed only while a policy is needed). */
int ss_hook_set_mode(int mode);
/* The training loop says where it is: 0 forward, 1 backward, 2 optimizer (goes into sig >> 16). */
int ss_hook_set_phase(uint32_t phase);
/* ss_trace_begin on the hooked context, event ids restart at 0, phase 0. */
int ss_hook_begin_iteration(void);
/* Unregister the operator callback and forget the context. */
int ss_hook_remove(void);
/* Detailed mode's tensor table of the current iteration (Sec. 3: per tensor its pointer, type and
 * uses): one row per block the allocator handed out since ss_hook_begin_iteration, in allocation
 * order (tensor_id = the id of its events).  producer_op / alloc_op = the operator running when it was
 * allocated, out_slot = its rank among that operator's allocations, dtype = type code of the first
 * output tensor seen in it, last_fwd_use = the last forward-phase operator that had it among its
 * inputs (the producer if none; SS_NONE_OP for blocks allocated after the forward phase),
 * first_bwd_use = the first later-phase operator that had it among its inputs (else SS_NONE_OP),
 * free_op = the operator running when it was released (the last operator if it is still held),
 * nbytes = the size asked for; offsets are 0.  In: *n = capacity, out: count; SS_E_CAPACITY with
 * the needed count in *n if out is too small. */
int ss_hook_tensor_table(ss_tensor_t *out /* host */, uint32_t *n);
/* For an executor that runs inside the framework (Sec. 5: the swaps of a policy are issued at their
 * operators of the running iteration; Sec. 5.1: a policy tensor is known by its producing operator and
 * output slot).  ss_hook_current_op: the number of operators recorded so far in this iteration, i.e. the
 * index the next dispatched operator will get.  ss_hook_block_of (Detailed mode): the tensor-table row, as
 * filled so far, of the block of this iteration that contains device address dev_addr, and the block's
 * start address (nullable); SS_E_INVAL if the address lies in no block allocated since
 * ss_hook_begin_iteration (parameters, optimizer state, blocks of earlier iterations). */
int ss_hook_current_op(uint32_t *n_ops /* host, out */);
/* ss_hook_pause(1) ... ss_hook_pause(0) bracket work the executor does through the framework itself (views
 * of a tensor it keeps, the block it asks the allocator for): operators dispatched in between are not
 * recorded, so that the model's operators keep the indices the policy was made for, and blocks allocated in
 * between get out_slot SS_NONE_OP and leave the running operator's slot count alone (their alloc / free
 * events are recorded as usual).  Nests; SS_E_STATE on a resume without a pause. */
int ss_hook_pause(int on);
int ss_hook_block_of(const void *dev_addr /* device address, not dereferenced */, ss_tensor_t *row /* host, out */,
                     uint64_t *block_addr /* host, out, nullable */);
int ss_hook_get_stats(ss_hook_stats_t *out /* host, out */);

#ifdef __cplusplus
}
#endif
#endif
