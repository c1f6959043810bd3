/*
 * ss.h - C ABI of the swap-executor hot path for AMD Instinct MI355X (gfx950).
 *
 * The library implements the policy-application side of swap-based memory
 * optimisation for eager-mode LLM training (SmartSwap, arXiv 2509.11076):
 * recording an iteration as integers (Sec. 3), scanning the memory timeline
 * with and without a policy (Sec. 3 last paragraph, Sec. 4.2), comparing and
 * re-anchoring operator sequences (Sec. 3 Algo. 1, Sec. 5.1), turning a policy
 * into the iteration's swap schedule (Sec. 5 first paragraph, Sec. 4.3), and
 * moving the selected activation tensors HBM -> pinned host memory -> HBM on
 * dedicated streams with device-side ordering against the compute stream
 * (Sec. 5.2).
 *
 * Conventions
 *  - Plain C, no exceptions cross the boundary.  Every function returns SS_OK
 *    (0) or a negative SS_E_* code; ss_strerror() names it; the last HIP error
 *    code is kept in the statistics.  A failed host allocation inside the
 *    library comes back as SS_E_NOMEM.
 *  - "host" pointers are ordinary process memory owned by the caller and only
 *    read or written during the call.  "device" pointers are HBM addresses.
 *    The library never allocates or frees the caller's device arena.
 *  - The library owns: pinned host staging, its streams and events, device
 *    copies of descriptor tables, scratch for the scan / match kernels, and the
 *    pinned trace arrays.
 *  - One ss_ctx per GPU; calls on one ctx come from one host thread.
 *  - All results are integers or bytes.
 */
#ifndef SS_H
#define SS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ss_ctx ss_ctx;

/* ---- error codes --------------------------------------------------------- */
enum {
  SS_OK = 0,
  SS_E_INVAL = -1,      /* bad argument (null pointer, out-of-range index, overflow risk) */
  SS_E_NOMEM = -2,      /* host, pinned or device allocation failed / staging too small */
  SS_E_HIP = -3,        /* a HIP call failed; code in ss_stats_t.last_hip_error */
  SS_E_INFEASIBLE = -4, /* no candidate left although memory still exceeds the budget (Algo. 2) */
  /* -5 and -7 are not used */
  SS_E_ORDER = -6,      /* events not in operator order where that is required */
  SS_E_STATE = -8,      /* call out of sequence (e.g. swap before a schedule is loaded) */
  SS_E_CAPACITY = -9,   /* a caller-provided output array or a configured maximum is too small */
  SS_E_TIMEOUT = -10    /* SS_CFG_BARE_RING: a stream gave up waiting for a ring transfer (flag_wait_ms); the
                           bytes moved in this iteration are not to be trusted */
};

/* ---- records (all little-endian, naturally aligned, no padding) ---------- */

/* One dispatched operator (Sec. 3).  op_token: dense id of the operator name,
 * 1.. in first-seen order, 0 = padding.  stack_hash: 32-bit FNV-1a of the
 * call-stack string, computed when the string is first seen.  sig: data-type
 * code | (n_out & 0xff) << 8 | phase << 16 (phase 0 forward, 1 backward, 2
 * optimizer).  n_out: number of output tensors. */
typedef struct { uint32_t op_token, stack_hash, sig, n_out; } ss_op_t;            /* 16 B */

/* One allocation (delta > 0) or release (delta < 0) of the memory trace,
 * caused by operator op_idx (Sec. 3, last paragraph). */
typedef struct { uint32_t op_idx, tensor_id; int64_t delta; } ss_event_t;         /* 16 B */

#define SS_NONE_OP 0xFFFFFFFFu

/* One tensor of the current iteration.  last_fwd_use / first_bwd_use are
 * SS_NONE_OP when there is none.  dev_off is the block's offset in the bound
 * arena from allocation until it is released; dev_off_in the offset of the
 * block the tensor is swapped back into (may differ). */
typedef struct {
  uint32_t tensor_id, dtype, producer_op, out_slot;
  uint32_t alloc_op, last_fwd_use, first_bwd_use, free_op;
  uint64_t dev_off, dev_off_in, nbytes;
} ss_tensor_t;                                                                     /* 56 B */

/* Identity of a policy tensor: output slot out_slot of operator ref_op of the
 * sequence the policy was generated for (Sec. 5.1). */
typedef struct { uint32_t ref_op, out_slot; } ss_anchor_t;                        /* 8 B */

/* One policy item (Sec. 4.3, 4.4): identity plus the four points.  As input
 * only ref_op, out_slot, tensor_id and nbytes are read; ss_apply_policy fills
 * the rest for the current iteration. */
typedef struct {
  uint32_t ref_op, out_slot, tensor_id, flags;
  uint32_t t_out;   /* swap-out is issued after this operator (last forward use)            */
  uint32_t t_free;  /* block is released after dispatching this operator (Sec. 5.2)          */
  uint32_t t_in;    /* swap-in is issued before this operator (pre-trigger, Sec. 4.3.1)     */
  uint32_t t_use;   /* first backward use: compute waits for the swap-in before it          */
  uint64_t nbytes;
} ss_policy_item_t;                                                                /* 40 B */
enum { SS_F_UNMATCHED = 1, SS_F_ORDER = 2, SS_F_LATE = 4, SS_F_RESIZED = 8, SS_F_FORCED = 16 };

/* One copy: nbytes between arena + dev_off and staging + host_off. */
typedef struct { uint64_t dev_off, host_off, nbytes; uint32_t tensor_id, flags; } ss_desc_t; /* 32 B */

/* One scheduled action.  Inside one operator index the order is
 * IN, WAIT_IN, [the operator itself], OUT, FREE. */
enum { SS_ACT_IN = 0, SS_ACT_WAIT_IN = 1, SS_ACT_OUT = 2, SS_ACT_FREE = 3 };
typedef struct { uint32_t op_idx, kind, tensor_id, batch; } ss_action_t;          /* 16 B */

/* ---- configuration -------------------------------------------------------- */
enum { SS_PATH_AUTO = 0, SS_PATH_KERNEL = 1, SS_PATH_ENGINE = 2,
       SS_PATH_STAGED = 3 };  /* through a ring in HBM.  Swap-out: the copy kernel gathers consecutive batches into
                                 a ring slot (their blocks can be released as soon as that is done) and one
                                 copy-engine transfer per slot carries them to the staging area.  Swap-in: one
                                 copy-engine transfer brings the staging range of several consecutive batches
                                 into a ring slot, issued with the first of them (so the link runs ahead of the
                                 blocks becoming free), and the copy kernel scatters each batch into its blocks at
                                 the batch's own issue point.  Used for batches whose staging slots are gap-free
                                 (sizes multiples of `align`, no guards) and fit a ring slot; other batches
                                 move as with SS_PATH_AUTO                                                   */
enum { SS_CFG_TIMING = 1,        /* record start/stop events per batch (ss_batch_ms)          */
       SS_CFG_POISON_FREE = 2,   /* overwrite a block with 0xDB when its FREE action runs     */
       SS_CFG_KEEP_LATE = 4,     /* keep items whose swap-out cannot finish before their first
                                    backward use (released and re-fetched around that use, the
                                    compute stream waiting) instead of dropping them            */
       SS_CFG_SYSTEM_FENCE = 8,  /* ordering events carry a system-scope fence (default: device
                                    scope; the host reads staging only after a synchronisation) */
       SS_CFG_POLICY_POINTS = 16,/* ss_apply_policy keeps each item's own t_free / t_in (as made by
                                    ss_generate_policy), moved along with the tensor's last forward /
                                    first backward use, instead of re-timing with the link model  */
       SS_CFG_STALL_TIMING = 32, /* measurement mode: one more event on the compute stream before every
                                    device-side wait, and SS_SYNC_DRAIN also waits for the compute stream
                                    and adds the waits' durations to ss_stats_t.stall_*_ms          */
       SS_CFG_MEMORY_MARKERS = 128, /* where a batch moved by a kernel (copy kernel, gather, scatter) has to be
                                    ordered after the compute stream's position, that position is published by a
                                    one-thread kernel on the compute stream that stores a running count in
                                    device memory, and the swap stream waits for the count in a one-wave kernel
                                    (bounded by flag_wait_ms, SS_E_TIMEOUT at the end of the iteration), instead
                                    of an event recorded on the compute stream that the swap stream waits for:
                                    such an event costs the compute stream 0.13 ms each time here, the kernel a
                                    few microseconds.  Batches moved by copy engine keep the event               */
       SS_CFG_BARE_RING = 64 };  /* SS_PATH_STAGED: the copy-engine transfers out of and into the rings are
                                    enqueued with nothing before and nothing behind them on their stream
                                    but other such transfers.  A copy-engine transfer that shares its stream
                                    with an event record or a wait slows the kernels of every other stream
                                    by 11-16 % for as long as it runs; a stream of transfers only does
                                    not.  So a thread of the library's own holds each transfer back on the
                                    host until what it has to wait for is complete, and its completion is
                                    published by a second small transfer behind it that writes a sequence
                                    number into device memory; a stream that needs the transfer's bytes
                                    waits for that number in a one-wave kernel which polls it, sleeping in
                                    between, and gives up after flag_wait_ms (SS_SYNC_DRAIN then returns
                                    SS_E_TIMEOUT).  The transfers themselves carry no events: with
                                    SS_CFG_TIMING their durations (ss_batch_ms, directions 2 and 3) are taken
                                    on the host's clock by a second thread that watches a copy of the
                                    sequence number arrive in pinned memory, and ss_batch_window has none
                                    for them (SS_E_STATE).  Batches that do not go through a ring then move
                                    by copy kernel, never by copy engine, and the caller should not enqueue
                                    copy-engine transfers of its own behind waits for swapped-in tensors: a
                                    transfer whose turn has not come holds up the engine's queue, in which
                                    the sequence numbers travel (the waits are bounded, so the worst case is
                                    SS_E_TIMEOUT).  Without SS_PATH_STAGED the flag does nothing            */

typedef struct {
  uint64_t staging_bytes;     /* pinned host staging to allocate at ss_create                */
  uint64_t link_bytes_per_op; /* link model: bytes the host link moves during one operator
                                 (Eq. 3 with Eq. 1 at one operator per group); >= 1           */
  uint64_t prefetch_bytes_per_op; /* same for the swap-in queue only (0 = link_bytes_per_op); a smaller
                                 value pre-triggers swap-ins with more margin (Sec. 4.3.1)       */
  uint64_t engine_min_bytes;  /* SS_PATH_AUTO: swap-in batches whose mean tensor size reaches this go to
                                 the copy engine, smaller ones to the copy kernel (default 4 MiB) */
  uint32_t align;             /* staging slot alignment, power of two >= 16 (default 256)    */
  uint32_t guard_bytes;       /* untouched bytes before/after each staging slot (mult. of align) */
  uint32_t stage_m, stage_n;  /* Algo. 1 hyper-parameters (defaults 2, 5)                    */
  uint32_t copy_path;         /* SS_PATH_* for swap-out batches                              */
  uint32_t copy_path_in;      /* SS_PATH_* for swap-in batches                               */
  uint32_t copy_workgroups;   /* grid size of the copy kernels (0 = default)                 */
  uint32_t copy_workgroups_out; /* grid size of the swap-out copy kernel (0 = copy_workgroups) */
  uint32_t copy_unroll;       /* 16-byte accesses in flight per lane: 2, 4 or 8 (0 = 8)      */
  uint32_t max_ops;           /* trace capacity in operators                                 */
  uint32_t max_events;        /* trace capacity in events                                    */
  uint32_t flags;             /* SS_CFG_*                                                    */
  uint64_t engine_min_bytes_out; /* SS_PATH_AUTO: the same for swap-out batches (default 32 MiB: below
                                 that the copy engine falls far behind the link inside a running
                                 training step, above it it reaches the link peak and, unlike a copy
                                 kernel, does not delay the compute stream's launches); 0 = never   */
  uint32_t out_streams;       /* streams the copy-kernel swap-out batches take in turn, 1..4 (0 = 1).  More than
                                 one lets a launch's set-up hide behind the launch before it, but every stream
                                 beyond the process's hardware queues (4 here, the compute stream included)
                                 shares a queue with another and waits for that one's work            */
  uint32_t in_streams;        /* the same for copy-kernel swap-in batches (0 = 1); copy-engine batches of
                                 either direction always use one stream                            */
  uint64_t ring_bytes;        /* SS_PATH_STAGED: size of the HBM ring of a direction (0 = 1 GiB), allocated at
                                 ss_create, one per staged direction                                          */
  uint64_t ring_slot_bytes;   /* SS_PATH_STAGED: size of one ring slot = largest single transfer (0 = 256 MiB:
                                 transfers of 64-134 MB out of the ring were seen to fall to a quarter of the
                                 link rate for four transfers in a row, 252 MB and larger never)              */
  uint32_t gather_workgroups; /* SS_PATH_STAGED: grid of the gather launches, HBM to HBM (0 = 256)          */
  uint32_t ring_taper;        /* SS_PATH_STAGED: 0 = group sizes are tapered at the ends of the iteration: the first
                                 swap-out groups and the first swap-in groups grow from an eighth of a slot by
                                 doubling (the first transfer leaves after a little of the forward pass instead
                                 of a slot's worth; the backward pass resumes after the first small transfer),
                                 and the last swap-in groups shrink (each at most half of what is still to come,
                                 down to an eighth of a slot), so that little of the backward pass is left to
                                 compute once the last transfer is back; a single batch is never split;
                                 1 = every group as large as a slot allows; n = 2..16 = as 0, but a last swap-in
                                 group takes at most 1/n of what is still to come: where the operators that use
                                 a group take a fraction r of the time the link needs for the next one, groups
                                 that halve arrive faster than they are used up and the work piles up behind the
                                 last one; n >= 1 / (1 - r) keeps the compute stream level with the link       */
  uint32_t copy_desc_lookup;  /* how a workgroup of the copy kernel finds the tensor a chunk belongs to: 0 = a
                                 per-chunk index table in global memory (4 bytes per chunk, built when the
                                 schedule is loaded; no search, no barrier), 1 = the batch's chunk-prefix table
                                 staged in LDS and searched per chunk (batches of up to 8,191 tensors; longer
                                 ones take the table).  Same bytes either way; 0 is faster on small tensors  */
  uint32_t copy_cus;          /* 0 = the swap streams' kernels may run on every compute unit; n > 0 = only on n of
                                 them (a compute-unit mask on those streams, spread over the dies), so that the
                                 copy kernel's long-lived waves occupy those units and no others.  The runtime
                                 creates such streams in its blocking form only: they synchronise with the null
                                 stream, so the compute stream bound must be another one.  Measured: masks of 8
                                 to 64 units do not change what a link-saturating copy kernel costs the compute
                                 stream; kept for measurement                                                */
  uint32_t engine_window_in;  /* copy-engine swap-in batches outstanding at most (0 = no limit): ss_swap_in returns
                                 only once the engine swap-in batch issued this many batches earlier has finished.
                                 Copy-engine transfers queued behind more than a few others run at a fraction of
                                 the link rate; the dispatch thread waits only where the compute stream is waiting
                                 for the same transfers                                                      */
  uint32_t engine_window_out; /* the same for copy-engine swap-out batches and ss_swap_out                     */
  uint32_t flag_wait_ms;      /* SS_CFG_BARE_RING, SS_CFG_MEMORY_MARKERS: longest a stream polls for a sequence number before it
                                 gives up and goes on, in ms (0 = 10,000; at most 600,000).  Once one wait has given
                                 up, no later wait of the iteration polls at all                            */
  uint32_t reserved0;
} ss_config_t;

/* ---- results ---------------------------------------------------------------- */
typedef struct {
  int64_t peak;        /* largest memory in use at any operator (>= base)                   */
  int64_t final_total; /* total after the last event (== base for a balanced iteration)     */
  int32_t argpeak_op;  /* first operator attaining the peak, -1 if there are no operators   */
  uint32_t n_over;     /* operators whose memory exceeds the budget (length of the MRL)     */
  uint32_t sorted;     /* 1 if both event lists were in operator order                      */
  uint32_t reserved;
} ss_scan_result_t;

enum { SS_STAGE_WARMUP = 0, SS_STAGE_GENPOLICY = 1, SS_STAGE_STABLE = 2 };
enum { SS_MATCH_STEP_STAGE = 1,  /* advance the Algo. 1 stage machine with this verdict      */
       SS_MATCH_HISTOGRAM = 2,   /* cosine of per-token occurrence counts instead of positions */
       SS_MATCH_ALIGN = 4 };     /* anchors land where the alignment of the two sequences pairs their
                                    operator (as ss_align_sequence), level SS_LEVEL_ALIGN           */
enum { SS_LEVEL_ALIGN = 3 };
typedef struct {
  uint64_t dot, na, nb;   /* integer sums of the cosine (na: current, nb: reference)        */
  uint32_t similar;       /* 1 if length differs by < 5 % and cosine > 95 %                 */
  uint32_t stage;         /* stage after this call (unchanged without SS_MATCH_STEP_STAGE)  */
  uint32_t stable_step;   /* Algo. 1 counter after this call                                */
  uint32_t n_unmatched;   /* anchors with new_idx == -1                                     */
} ss_match_result_t;

typedef struct {
  uint32_t lcs;           /* length of the longest common subsequence                       */
  uint32_t distance;      /* insertions + deletions turning ref into cur: n + m - 2 lcs     */
  uint32_t n_keys;        /* distinct (op_token, stack_hash, sig) in cur                    */
  uint32_t n_unmatched;   /* anchors with new_idx == -1                                     */
} ss_align_result_t;

typedef struct {
  uint64_t staging_bytes;   /* staging the schedule needs                                    */
  uint64_t bytes_out;       /* sum of nbytes over swap-out descriptors (== swap-in)         */
  uint32_t n_kept, n_dropped, n_late;
  uint32_t n_out_batches, n_in_batches, reserved;
} ss_apply_result_t;

typedef struct {
  uint64_t bytes_out, bytes_in;         /* since ss_create                                  */
  uint64_t kernel_batches, engine_batches;
  uint64_t free_waits, in_waits;        /* device-side stream waits issued for FREE / WAIT_IN */
  uint64_t ops_recorded, events_recorded;
  int32_t last_hip_error;               /* hipError_t of the last failing HIP call, 0 if none */
  uint32_t engine_batches_out;          /* of engine_batches, the swap-out ones             */
  /* anchors placed by ss_match_sequence / ss_align_sequence since ss_create, by the level that placed
   * them: [0] (token, stack, sig), [1] (token, sig), [2] (token), [3] sequence alignment, [4] unmatched */
  uint64_t match_levels[5];
  /* memory-block reuse interval of the loaded schedule (Sec. 6.4): per swapped tensor the number of
   * operators between issuing its swap-out and releasing its block (t_free - t_out); bucket b counts
   * the tensors with floor(log2(interval + 1)) == b (b = 15: that or more); sum and count give the mean */
  uint32_t reuse_hist[16];
  uint64_t reuse_sum, reuse_count;
  /* with SS_CFG_STALL_TIMING: time the compute stream spent inside the device-side waits of
   * SS_SYNC_FREE / SS_SYNC_WAIT_IN (from the moment it reached the wait to the end of the batch it
   * waited for, 0 if that had already ended), summed over the iterations drained so far */
  double stall_free_ms, stall_wait_in_ms;
  uint64_t ring_batches, ring_transfers; /* SS_PATH_STAGED: swap-out batches gathered into the HBM ring, and
                                            copy-engine transfers that carried them out of it */
  uint64_t ring_batches_in, ring_transfers_in; /* the same for swap-in: batches scattered out of the ring, transfers into it */
  uint64_t engine_window_waits;         /* times ss_swap_in / ss_swap_out waited for an earlier engine batch (engine_window_*) */
} ss_stats_t;

typedef struct {
  double d2h_gbps, h2d_gbps;            /* one direction at a time                          */
  double bidir_d2h_gbps, bidir_h2d_gbps;/* both directions at once, per direction           */
  double kernel_d2h_gbps, kernel_h2d_gbps; /* same buffers through the copy kernels         */
  double kernel_bidir_d2h_gbps, kernel_bidir_h2d_gbps; /* copy kernels, both directions at once */
} ss_bw_t;

/* ---- life cycle -------------------------------------------------------------- */

/* Fill *cfg with defaults (staging 64 MiB, link 64 MiB/op, align 256, no guard, m=2, n=5,
 * auto paths, 65536 operators, 1048576 events). */
int ss_config_default(ss_config_t *cfg /* host, out */);

/* Create a context on the current HIP device: allocates pinned staging and pinned trace arrays and takes
 * the swap-out / swap-in (/ ring-transfer) streams (Sec. 5.2: the swaps run on streams of their own).
 * The streams are non-blocking, at the default priority, and kept for the life of the process: ss_destroy
 * hands them to the next context that asks for the same role, so every context of a process runs on the
 * streams the first one got (where the runtime places a new stream changes how much a transfer costs the
 * kernels beside it; streams with a compute-unit mask, copy_cus > 0, are the context's own).  Contexts
 * alive at the same time get different streams.
 * With SS_CFG_BARE_RING and a ring route the context also starts a host thread of its own that issues the
 * ring transfers (and, with SS_CFG_TIMING, a second one that watches them complete); both end in ss_destroy.
 * The calls on one context still have to come from one thread at a time.
 * SS_E_NOMEM if pinned memory is refused. */
int ss_create(ss_ctx **out /* host, out */, const ss_config_t *cfg /* host, nullable */);
int ss_destroy(ss_ctx *ctx);

/* Bind the caller's device arena [arena, arena + arena_bytes) and the compute
 * stream (a hipStream_t, e.g. torch.cuda.Stream.cuda_stream; NULL = the null
 * stream).  Every dev_off is relative to `arena`.  May be called again.
 * arena = NULL with arena_bytes = 0 binds no arena: see ss_swap_out_from. */
int ss_bind(ss_ctx *ctx, void *arena /* device */, uint64_t arena_bytes, void *compute_stream);

/* ---- a1: trace record (Sec. 3) ------------------------------------------------ */

/* Reduce an operator's strings to integers, once: token of `name` (dense,
 * first-seen order), FNV-1a hash of `stack`, signature.  The hot path below
 * never sees a string (Sec. 5.1). */
int ss_intern_op(ss_ctx *ctx, const char *name, const char *stack, uint32_t dtype,
                 uint32_t n_out, uint32_t phase, ss_op_t *out /* host, out */);

/* Start recording a new iteration (the previous one is dropped). */
int ss_trace_begin(ss_ctx *ctx);

/* Append one dispatched operator and the n_ev alloc/free events it caused.
 * Every event's op_idx must equal the index of this operator; token 0 is
 * refused.  SS_E_CAPACITY beyond max_ops / max_events. */
int ss_trace_record(ss_ctx *ctx, const ss_op_t *op /* host */, const ss_event_t *ev /* host, nullable */,
                    uint32_t n_ev);

/* For dispatch hooks that learn things only after the operator has been recorded (its outputs
 * when it returns, the allocator's calls while it runs; Sec. 3 Detailed mode):
 * ss_trace_event appends one alloc (+) / free (-) event to the most recently recorded operator
 * (SS_E_ORDER before the first operator of the iteration, SS_E_CAPACITY beyond max_events);
 * ss_trace_amend sets the data-type code and output count of recorded operator op_idx (the
 * phase and the token stay). */
int ss_trace_event(ss_ctx *ctx, uint32_t tensor_id, int64_t delta);
int ss_trace_amend(ss_ctx *ctx, uint32_t op_idx, uint32_t dtype, uint32_t n_out);

/* Borrow the recorded arrays (valid until the next ss_trace_begin / ss_destroy)
 * and the running sum of all deltas (0 for a balanced iteration). */
int ss_trace_view(ss_ctx *ctx, const ss_op_t **ops, uint32_t *n_ops, const ss_event_t **ev,
                  uint64_t *n_ev, int64_t *balance);

/* ---- a2: timeline scan (Sec. 3 last paragraph, Sec. 4.2) ---------------------- */

/* Memory in use per operator from the alloc/free trace `ev` and, optionally,
 * the policy-induced events `pev` (a release of nbytes at t_free, an allocation
 * at t_in per swapped tensor).  Memory at operator t is what was held on entry
 * plus everything t allocates; what t releases goes when t ends; a policy
 * allocation comes first in its operator and a policy release last.
 *   per_op[t] = base + sum(delta of operators < t) + sum(positive delta of t)
 *   mre[t]    = max(0, per_op[t] - budget)      (memory reduction entries)
 * timeline (nullable, n_ev + n_pe entries) receives the running total after
 * each event in canonical order (operator, class, position in own list; class 0
 * policy alloc, 1 trace alloc, 2 trace release, 3 policy release); it needs both
 * lists in operator order, else SS_E_ORDER (other outputs are still valid).
 * All arrays are host memory; per_op / mre (nullable) have n_ops entries.
 * SS_E_INVAL if an event names an operator >= n_ops. */
int ss_timeline_scan(ss_ctx *ctx, const ss_event_t *ev, uint64_t n_ev,
                     const ss_event_t *pev /* nullable */, uint64_t n_pe, uint32_t n_ops,
                     int64_t base, int64_t budget, int64_t *timeline, int64_t *per_op,
                     int64_t *mre, ss_scan_result_t *res /* host, out */);

/* k scans of the same trace, each under its own policy events, in one kernel launch (one
 * workgroup per scan): candidate policies are checked against the memory limit together
 * (Sec. 4.4 generates several policies and keeps one).  pev holds the k lists back to back,
 * list c being pev[pe_start[c] .. pe_start[c+1]) (pe_start has k + 1 entries, pe_start[0] = 0);
 * res has k entries; per_op (nullable) k * n_ops entries, scan c at per_op + c * n_ops.  Same
 * definitions and errors as ss_timeline_scan; no timeline.  k <= 4096.  Host memory. */
int ss_timeline_scan_batch(ss_ctx *ctx, const ss_event_t *ev, uint64_t n_ev, const ss_event_t *pev,
                           const uint64_t *pe_start, uint32_t k, uint32_t n_ops, int64_t base,
                           int64_t budget, int64_t *per_op, ss_scan_result_t *res /* host, out */);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): the scan of ss_timeline_scan with nothing allocated, copied or waited
 * for.  Inputs and outputs are the caller's DEVICE arrays (same meaning, sizes and nullability as
 * above; d_res is required); the kernel's scratch is a static device array of 9.75 MiB that every GPU
 * the library runs on holds until the process ends.  The call enqueues one kernel (three from 32,768 events on) on `stream` (a
 * hipStream_t of the context's device, which must be current; NULL = the null stream) and returns;
 * results are valid once that stream has reached the kernel's end.
 * Limits: n_ops <= 65,536 and n_ev + n_pe <= 262,144, else SS_E_CAPACITY (nothing is enqueued).
 * Errors the kernel finds are reported in d_res->reserved: bit 0 = an event names an operator
 * >= n_ops (no other output is meaningful), bit 1 = a list is not in operator order (d_res->sorted
 * is 0 and the timeline is not written; the other outputs are valid).
 * All calls on one GPU share the one scratch array: calls that overlap in time on the same GPU
 * (different streams, different contexts) race; the kernel clears what it needs itself, so calls
 * in sequence need nothing between them. */
int ss_timeline_scan_static(ss_ctx *ctx, void *stream, const ss_event_t *d_ev /* device */, uint64_t n_ev,
                            const ss_event_t *d_pev /* device, nullable */, uint64_t n_pe, uint32_t n_ops,
                            int64_t base, int64_t budget, int64_t *d_timeline /* device, nullable */,
                            int64_t *d_per_op /* device, nullable */, int64_t *d_mre /* device, nullable */,
                            ss_scan_result_t *d_res /* device, out */);

/* ---- a3: sequence match (Sec. 3 Algo. 1, Sec. 5.1) ---------------------------- */

/* (i) Similarity of the current sequence `cur` to `ref`: similar iff
 * 20 * |m - n| < n and cosine > 0.95, the cosine taken positionally with the
 * shorter sequence zero-padded, evaluated exactly in integers
 * (400 dot^2 > 361 na nb, dot > 0).  With SS_MATCH_STEP_STAGE the Algo. 1 stage
 * machine (m, n from the configuration) advances with the verdict.
 * (ii) For each anchor the operator index in `cur` that corresponds to
 * operator ref_op of `ref`: keyed-ordinal matching, relaxing the key from
 * (token, stack, sig) to (token, sig) to (token); a landing place must have
 * more than out_slot outputs and the same data-type code; among anchors landing
 * on the same (operator, slot) the lowest anchor index keeps it.
 * new_idx[k] (int32, -1 = none) and level[k] (0..2, 255 = none) are host arrays.
 * Limits: tokens < 2^18, n, m <= 2^23 (keeps the sums below 2^59). */
int ss_match_sequence(ss_ctx *ctx, const ss_op_t *ref, uint32_t n, const ss_op_t *cur, uint32_t m,
                      const ss_anchor_t *anchors /* nullable if k == 0 */, uint32_t k, uint32_t flags,
                      int32_t *new_idx, uint8_t *level, ss_match_result_t *res /* host, out */);

/* Align the current sequence with the reference one as a whole (Sec. 5.1: identification must
 * survive minor variations of the sequence; the paper gives no algorithm, this is the build's).
 * Two operators are equal when (op_token, stack_hash, sig) are equal.  The longest common
 * subsequence is computed on the GPU; of the optimal alignments the one read from the end of both
 * sequences is taken: equal operators pair, otherwise step back in cur if that loses nothing, else
 * in ref.  ref_to_cur[i] (nullable, n_ref entries) = operator of cur paired with ref[i], or -1.
 * An anchor lands on the operator its ref_op is paired with if that operator has more than
 * out_slot outputs (level SS_LEVEL_ALIGN), else -1 / 255.  Unlike the keyed ordinals of
 * ss_match_sequence this does not misland when an operator with the anchor's own key was dropped or
 * inserted earlier in the sequence.  Limits: n_ref, n_cur <= 65536 and n_ref * ceil(n_cur / 64) * 8
 * bytes <= 1 GiB (SS_E_CAPACITY).  All arrays are host memory. */
int ss_align_sequence(ss_ctx *ctx, const ss_op_t *ref, uint32_t n_ref, const ss_op_t *cur, uint32_t n_cur,
                      const ss_anchor_t *anchors /* nullable if n_anchors == 0 */, uint32_t n_anchors,
                      int32_t *ref_to_cur, int32_t *new_idx, uint8_t *level,
                      ss_align_result_t *res /* host, out */);

/* ---- a4: apply policy (Sec. 5 first paragraph; Sec. 4.3 timing) ---------------- */

/* Resolve each policy item against this iteration's tensor table (the output
 * slot out_slot of operator new_idx[a]), take t_out / t_use from the current
 * tensor, time release and pre-trigger with the FIFO link model
 * (link_bytes_per_op for the swap-out queue, prefetch_bytes_per_op for the swap-in queue;
 * no swap-in is issued before the last swap-out of the set), drop what is unmatched or has
 * no room (or keep it forced around its use with SS_CFG_KEEP_LATE), and build:
 *   resolved[k]  (nullable) the items with their points and flags filled in
 *   actions[*n_actions]     sorted by (operator, kind, queue rank); in: capacity, out: count (4 per kept item)
 *   descs_out / descs_in    one descriptor per kept item in swap-out / swap-in issue order (capacity k);
 *                           a swap-out batch = items issued after the same operator, a swap-in batch =
 *                           items issued before the same operator and first used by the same operator
 *   pevents[*n_pe]          policy events for ss_timeline_scan; in: capacity, out: count (2 per kept item)
 * and load the schedule into the context (as ss_load_schedule would).
 * Staging offsets are the exclusive prefix sum of align_up(nbytes, align) +
 * guard in swap-out order.  All arrays are host memory. */
int ss_apply_policy(ss_ctx *ctx, const ss_policy_item_t *policy, uint32_t k, const int32_t *new_idx,
                    const ss_tensor_t *tensors, uint32_t n_tensors, ss_policy_item_t *resolved,
                    ss_action_t *actions, uint32_t *n_actions, ss_desc_t *descs_out,
                    ss_desc_t *descs_in, ss_event_t *pevents, uint32_t *n_pe,
                    ss_apply_result_t *res /* host, out */);

/* Host-side, non-blocking: has swap-out (dir 0) / swap-in (dir 1) batch `batch` of this iteration
 * finished?  *done = 1 / 0.  SS_E_STATE if it has not been issued.  This is the event query a
 * host-polled release (the stock recordStream of Sec. 5.2) performs at every allocation; the executor
 * itself never calls it. */
int ss_batch_done(ss_ctx *ctx, uint32_t dir, uint32_t batch, int *done /* host, out */);

/* Borrow the batch tables of the loaded schedule: starts have n_batches + 1
 * entries; in_dep[b] is the last swap-out batch swap-in batch b depends on. */
int ss_schedule_view(ss_ctx *ctx, const uint32_t **out_start, uint32_t *n_out_batches,
                     const uint32_t **in_start, uint32_t *n_in_batches, const uint32_t **in_dep);

/* Load a schedule given directly as descriptors and batch boundaries (host
 * arrays; out_start has n_out_batches + 1 entries, likewise in_start; in_dep
 * has n_in_batches entries or is NULL = each swap-in batch waits for all
 * swap-outs).  Every descriptor is checked against the arena and the staging
 * area, every pair of staging slots for overlap.  Requires ss_bind. */
int ss_load_schedule(ss_ctx *ctx, const ss_desc_t *descs_out, uint32_t n_out, const uint32_t *out_start,
                     uint32_t n_out_batches, const ss_desc_t *descs_in, uint32_t n_in,
                     const uint32_t *in_start, uint32_t n_in_batches, const uint32_t *in_dep);

/* Longest-idle-first stand-in for the policy generator (Algo. 2): add
 * candidates (kept from forward to backward, idle span covering an
 * over-budget operator, nbytes >= min_bytes) one at a time, longest idle span
 * first, re-time and re-scan until the peak fits the budget.  `initial`
 * (nullable) are items already in force.  policy_out receives the initial
 * items followed by the added ones; in: capacity *n_policy, out: count.
 * SS_E_INFEASIBLE when candidates run out. */
int ss_greedy_policy(ss_ctx *ctx, const ss_tensor_t *tensors, uint32_t n_tensors, const ss_event_t *ev,
                     uint64_t n_ev, uint32_t n_ops, int64_t base, int64_t budget, uint64_t min_bytes,
                     const ss_policy_item_t *initial, uint32_t n_initial,
                     ss_policy_item_t *policy_out, uint32_t *n_policy, int64_t *peak_out);

/* ---- policy generator (Sec. 4: Eq. 1-3, Algo. 2) ---------------------------------- */

typedef struct {
  uint32_t g_fwd, g_bwd;  /* number of logical layers the forward / backward operators are cut into */
  uint32_t c_num, c_den;  /* C of Eq. 2 as a fraction                                               */
  uint64_t min_bytes;     /* tensors smaller than this are never candidates                         */
  uint64_t phase_bytes_per_op[3]; /* Eq. 1 per phase: link bytes per forward / backward / optimizer
                             operator (link peak x that phase's measured time / its operator count);
                             0 = the context's link_bytes_per_op, i.e. Eq. 1 as printed          */
} ss_gen_params_t;

typedef struct {
  int64_t peak_no_swap;        /* timeline scan without a policy                                    */
  int64_t peak_with_policy;    /* timeline scan with the generated policy's own points              */
  uint32_t n_over_with_policy; /* operators still above the limit under that scan                   */
  uint32_t n_rounds;           /* passes of the Algo. 2 loop                                        */
  uint32_t n_items, n_late;
  uint64_t bytes;              /* sum of nbytes of the items                                        */
} ss_gen_result_t;

/* Generate a swap policy as Sec. 4 describes.  The memory without swaps comes from a timeline scan
 * of `ev`; every operator above `limit` gets a memory reduction entry; candidates (kept from
 * forward to backward, >= min_bytes, spanning at least one entry) are ranked by Eq. 2; the simulator
 * places each swap-in in a logical layer before the first backward use that still has time left
 * (Eq. 1 gives a layer link_bytes_per_op x its operator count, Eq. 3 makes a transfer cost its
 * size), never back into the peak period, subtracts the tensor from the entries it covers, and
 * repeats until no entry is left (SS_E_INFEASIBLE when candidates run out first); finally every
 * swap-out is given the first layer with time left from its last forward use on (of that use's own
 * layer only the operators after the use count: the swap-out starts there, Sec. 4.3.2), which fixes the
 * release point.  Operator phases are read from ops[].sig >> 16.
 * policy_out receives the items in the order they were committed, with t_out, t_free, t_in, t_use
 * filled (use SS_CFG_POLICY_POINTS to have ss_apply_policy keep them); in: capacity *n_policy,
 * out: count.  All arrays are host memory.
 * SS_OK does not by itself mean that the limit is kept: the simulator counts a tensor as gone from the
 * operator after its last forward use, the release point fixed afterwards may lie later, so the scan of
 * the finished policy (res->peak_with_policy, res->n_over_with_policy) can still show operators above
 * the limit.  A caller that must not exceed the limit checks res->n_over_with_policy == 0 and otherwise
 * lowers the limit, changes the parameters (ss_generate_policy_best ranks parameter sets by this count
 * first) or tops the policy up with ss_greedy_policy(initial = the generated items). */
int ss_generate_policy(ss_ctx *ctx, const ss_op_t *ops, uint32_t n_ops, const ss_tensor_t *tensors,
                       uint32_t n_tensors, const ss_event_t *ev, uint64_t n_ev, int64_t base, int64_t limit,
                       const ss_gen_params_t *params, ss_policy_item_t *policy_out, uint32_t *n_policy,
                       ss_gen_result_t *res /* host, out */);

/* Several parameter sets at once (Sec. 4.4 / Sec. 6: several policies are generated and one is
 * kept): one policy per set, all of them scanned with their own release / pre-trigger points in one
 * batched launch, and the best returned: no operator over the limit first (else fewest such
 * operators), then fewest LATE items, then fewest bytes, then the lowest index.  Sets for which the
 * generator runs out of candidates are skipped; SS_E_INFEASIBLE if that happens to all.
 * *chosen receives the index of the winning set, res its result. */
int ss_generate_policy_best(ss_ctx *ctx, const ss_op_t *ops, uint32_t n_ops, const ss_tensor_t *tensors,
                            uint32_t n_tensors, const ss_event_t *ev, uint64_t n_ev, int64_t base, int64_t limit,
                            const ss_gen_params_t *params, uint32_t n_params, ss_policy_item_t *policy_out,
                            uint32_t *n_policy, uint32_t *chosen, ss_gen_result_t *res /* host, out */);

/* ---- a5 / a6 / a7: swap-out, swap-in, release and wait (Sec. 5.2) --------------- */

/* Enqueue swap-out batch `batch`: the swap-out stream waits (on the device) for
 * everything enqueued so far on the compute stream, copies each tensor of the
 * batch to its staging slot and records the batch's done-event.  Returns at
 * once. */
int ss_swap_out(ss_ctx *ctx, uint32_t batch);

/* Enqueue swap-in batch `batch`: the swap-in stream waits for everything
 * enqueued so far on the compute stream (the destination blocks are free from
 * here on) and for the swap-out batches it depends on, copies each tensor
 * from its staging slot into its dev_off, records the done-event.  Swap-out batches are normally issued in
 * index order (ss_dispatch does); if they were not, the batch waits for every swap-out issued so far. */
int ss_swap_in(ss_ctx *ctx, uint32_t batch);

/* The same two moves for tensors whose device addresses are only known when the batch is issued: blocks
 * handed out by a framework's own allocator, as in the paper's setting, where the executor sits inside
 * the framework's dispatch path (Sec. 5) and a swapped-in tensor lands wherever the allocator puts it.
 * dev_src / dev_dst: host array with one device address per tensor of the batch, in the batch's descriptor
 * order (nullable for an empty batch); each address 16-byte aligned and valid for the descriptor's nbytes.
 * The descriptors' dev_off are replaced by these addresses for this and later iterations (relative to the
 * bound arena; ss_bind(ctx, NULL, 0, stream) binds no arena, the offsets are then the addresses
 * themselves, ss_load_schedule checks staging offsets only and the plain ss_swap_out / ss_swap_in refuse
 * non-empty batches with SS_E_STATE).  Such batches go by copy engine, which takes the addresses from the
 * host-side descriptors, unless the direction's path is SS_PATH_KERNEL: then the copy kernel gets the addresses as
 * launch arguments, one launch per tensor (on a real PyTorch bf16 model, copy-kernel launches beside the step
 * made the training loss irreproducible in the last bits in some runs although every byte moved was checked to
 * be right - as did the copy kernel moving an unrelated buffer with no ordering against the step: the model's
 * own kernels accumulate in an order that depends on what else holds compute units; with the copy engine every
 * run was bit-identical to no swapping).  Ordering, events, statistics and errors as ss_swap_out / ss_swap_in; SS_E_INVAL for a null or
 * misaligned address or one outside a bound arena; SS_E_STATE for a batch that belongs to a ring group
 * (SS_PATH_STAGED moves batches through rings by their arena offsets). */
int ss_swap_out_from(ss_ctx *ctx, uint32_t batch, const void *const *dev_src /* host array of device addresses */);
int ss_swap_in_to(ss_ctx *ctx, uint32_t batch, void *const *dev_dst /* host array of device addresses */);

enum { SS_SYNC_FREE = 0,    /* id = tensor: compute stream waits (device-side) for that tensor's
                               swap-out; after this call its block may be given to later operators */
       SS_SYNC_WAIT_IN = 1, /* id = tensor: compute stream waits (device-side) for its swap-in     */
       SS_SYNC_DRAIN = 2,   /* host waits for both swap streams; surfaces asynchronous errors      */
       SS_SYNC_ITERATION_END = 3 };
                            /* ends the iteration like SS_SYNC_DRAIN (batches may be issued again, the
                               other set of events is used) without making the host wait for it: the swap
                               streams' work of the next iteration is ordered behind this one's on the
                               device (staging slots and ring slots are not reused before their readers
                               are done).  The host waits only for the iteration BEFORE this one, so one
                               iteration at most is outstanding; what that one ran into (SS_E_HIP,
                               SS_E_TIMEOUT) is returned here, one call late.  A training loop whose host
                               thread runs ahead of the GPU keeps doing so (Sec. 5.2 asks the same of the
                               release of blocks); ss_host_peek and the timing calls want SS_SYNC_DRAIN
                               first.  With SS_CFG_STALL_TIMING, or SS_CFG_TIMING beside bare ring
                               transfers, the call is SS_SYNC_DRAIN                                    */
int ss_sync(ss_ctx *ctx, uint32_t what, uint32_t id);

/* The executor's step at one operator (Sec. 5, first paragraph): issues, in schedule order, every action that the schedule loaded by the last ss_apply_policy holds for
 * operator op_idx: when = 0, the ones that come before the operator is enqueued (SS_ACT_IN through
 * ss_swap_in once per batch, SS_ACT_WAIT_IN through ss_sync); when = 1, the ones that come after it
 * (SS_ACT_OUT through ss_swap_out once per batch, SS_ACT_FREE through ss_sync).  One call per side
 * of an operator replaces one call per action; an operator without actions costs a table lookup.
 * SS_E_STATE if no schedule made by ss_apply_policy is loaded (ss_load_schedule carries no actions),
 * SS_E_INVAL for when > 1; the first failing action's code otherwise (actions after it are not
 * issued). */
int ss_dispatch(ss_ctx *ctx, uint32_t op_idx, uint32_t when);

/* ---- support ------------------------------------------------------------------- */

/* Pointer into the pinned staging area (host) for checking results. */
int ss_host_peek(ss_ctx *ctx, uint64_t host_off, uint64_t nbytes, const void **ptr);
/* Fill the whole staging area with a byte (host side; for guard checks). */
int ss_staging_fill(ss_ctx *ctx, int byte);

/* Duration of a batch on its swap stream in ms (needs SS_CFG_TIMING), in the iteration drained last;
 * dir 0 = out, 1 = in, 2 = the copy-engine transfers out of the swap-out ring, 3 = those into the
 * swap-in ring (SS_PATH_STAGED; `batch` then counts the ring groups, see ss_ring_view).  A staged
 * batch's own duration is that of its gather into / scatter out of the ring.  span_ms (nullable): first start to last end over all batches (transfers)
 * of that direction. */
int ss_batch_ms(ss_ctx *ctx, uint32_t dir, uint32_t batch, float *ms, float *span_ms);

/* The same for every unit of a direction in one call: ms[u] = duration of unit u, or -1 if it did not
 * run that way in the iteration drained last (e.g. a ring group whose batches moved directly); in:
 * capacity of ms, *n out: number of units (SS_E_CAPACITY if it exceeds the capacity). */
int ss_batch_ms_all(ss_ctx *ctx, uint32_t dir, float *ms /* host, out */, uint32_t capacity, uint32_t *n);

/* Start and end of a batch on its swap stream, in ms since the start of swap-out batch 0 of
 * the same iteration (needs SS_CFG_TIMING; all batches involved must have completed). */
int ss_batch_window(ss_ctx *ctx, uint32_t dir, uint32_t batch, float *start_ms, float *end_ms);

/* SS_PATH_STAGED: how the loaded schedule's batches of direction dir (0 = out, 1 = in) were grouped.
 * n_groups ring groups; group_of (borrowed, one entry per batch of that direction) = the batch's group
 * or -1 if it moves directly; group_bytes (borrowed, n_groups entries) = bytes of each group's transfer. */
int ss_ring_view(ss_ctx *ctx, uint32_t dir, uint32_t *n_groups, const int32_t **group_of,
                 const uint64_t **group_bytes);

/* Host-link bandwidth measured now: pinned hipMemcpy D2H, H2D, both at once,
 * and the same through the copy kernels; `bytes` per transfer, median of `reps`. */
int ss_bw_probe(ss_ctx *ctx, uint64_t bytes, uint32_t reps, ss_bw_t *out /* host, out */);

int ss_get_stats(ss_ctx *ctx, ss_stats_t *out /* host, out */);
const char *ss_strerror(int code);
/* The last HIP failure seen by the calling thread (also when no context survived it):
 * returns the hipError_t, its name, and the library source position that saw it. */
int ss_last_hip_error(const char **name, const char **file, int *line);

#ifdef __cplusplus
}
#endif
#endif /* SS_H */
