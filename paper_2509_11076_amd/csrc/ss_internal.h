// Internal declarations shared by the translation units of libss.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <new>
#include <stdexcept>
#include <string>
#include <unordered_map>
#include <vector>

#include "ss.h"

// No C++ exception crosses the C boundary: an entry point that allocates host memory through the
// standard library runs its body inside this, and a failed allocation comes back as SS_E_NOMEM.
template <class Body>
inline int ss_guard(Body &&body) noexcept {
  try {
    return body();
  } catch (const std::bad_alloc &) {
    return SS_E_NOMEM;
  } catch (const std::length_error &) {
    return SS_E_NOMEM;
  } catch (...) {
    return SS_E_INVAL;
  }
}

struct ss_sched {
  std::vector<ss_desc_t> out, in;                 // host copies, issue order
  std::vector<uint32_t> out_start, in_start;      // batch boundaries (n_batches + 1)
  std::vector<uint32_t> in_dep;                   // per swap-in batch: last swap-out batch needed
  std::vector<uint32_t> out_chunk0, in_chunk0;    // per descriptor: first chunk index inside its batch
  std::vector<uint32_t> out_cdesc, in_cdesc;      // per chunk: descriptor index inside its batch
  std::vector<uint64_t> out_cbase, in_cbase;      // per batch: where its chunks start in *_cdesc
  std::vector<uint8_t> out_shift, in_shift;       // per batch: log2 of its chunk size
  std::unordered_map<uint32_t, uint32_t> out_of_tensor, in_of_tensor;  // tensor id -> descriptor index
  std::vector<uint32_t> out_batch_of, in_batch_of;                      // descriptor index -> batch
  std::vector<uint8_t> out_waited, in_waited, out_issued, in_issued;    // per batch, this iteration
  // Per-batch events exist twice: iterations alternate between the two sets (`phase`, switched by the
  // drain), so that the timing of the iteration drained last stays readable while the next one runs.
  std::vector<hipEvent_t> ev_out_done[2], ev_in_done[2], ev_out_start[2], ev_in_start[2];
  std::vector<hipEvent_t> ev_free_at, ev_wait_at;   // SS_CFG_STALL_TIMING: compute stream reaches the wait for the batch
  // Staged swap-out (SS_PATH_STAGED): consecutive batches whose staging slots form one gap-free range
  // are gathered by the copy kernel into a slot of the HBM ring and leave in one copy-engine transfer.
  struct out_group { uint32_t first, last; uint64_t host_lo, bytes; };
  std::vector<out_group> groups;
  std::vector<uint64_t> group_bytes;                // per group, for ss_ring_view
  std::vector<int32_t> group_of;                    // per swap-out batch: its group, -1 = leaves directly
  int64_t last_direct_out = -1;                     // swap-out batch that left directly (not through the ring) most recently, this iteration
  // swap-out batches issued out of index order (this iteration): a swap-in then waits for the batch issued most
  // recently on every swap-out stream instead of for the batches up to in_dep
  int64_t max_out_issued = -1;
  bool out_of_order = false;
  int64_t last_out_on[4] = {-1, -1, -1, -1};        // per swap-out stream: batch issued on it most recently
  std::vector<hipEvent_t> ev_gathered[2];           // per batch: its bytes are in the ring (the block may be released)
  std::vector<hipEvent_t> ev_flush_start[2];        // per group (SS_CFG_TIMING): its first transfer starts
  std::vector<int32_t> done_ev_of;                  // per batch, this iteration: batch whose ev_out_done covers it; -1 = not sent yet
  std::vector<int32_t> done_ev_of_drained;          // the same of the iteration drained last (for the timing calls)
  std::vector<uint8_t> ring_state;                  // per batch, this iteration: 0 not issued, 1 in the ring, 2 sent (or left directly)
  std::vector<uint32_t> group_pending;              // per group, this iteration: batches not issued yet
  std::vector<uint8_t> group_gathered, group_started; // per group: has bytes in the ring that are not sent; first transfer recorded
  std::vector<int32_t> group_last_flush_drained;    // the same of the iteration drained last
  std::vector<int32_t> group_last_flush;            // per group: batch whose ev_out_done its latest transfer recorded, -1 = none
  std::vector<int32_t> slot_owner;                  // per ring slot: group whose bytes it holds, -1 = none
  std::vector<uint8_t> out_staged_drained;          // the same of the iteration drained last
  std::vector<uint8_t> out_staged;                  // per batch, this iteration: it went through the ring
  int64_t last_gather_batch = -1;                   // batch gathered most recently (its event is the latest on the swap-out stream)
  int64_t last_flush_batch = -1;                    // batch whose ev_out_done the most recent transfer out of the ring recorded
  // Staged swap-in (copy_path_in = SS_PATH_STAGED): consecutive swap-in batches whose staging slots together
  // form one gap-free range come back in one copy-engine transfer into a slot of a second HBM ring, issued
  // with the group's first batch; each batch is then scattered from the ring into its blocks by the copy kernel
  // at its own issue point.
  struct in_group { uint32_t first, last; uint64_t host_lo, bytes; };
  std::vector<in_group> in_groups;
  std::vector<uint64_t> in_group_bytes;             // per group, for ss_ring_view
  std::vector<int32_t> in_group_of;                 // per swap-in batch: its group, -1 = comes back directly
  std::vector<std::vector<uint32_t>> in_group_outs; // per group: the swap-out batches its tensors left in
  std::vector<uint8_t> in_group_state;              // per group, this iteration: 0 untouched, 1 fetched, 2 not usable (direct)
  std::vector<int32_t> in_group_last_scatter;       // per group, this iteration: swap-in batch scattered most recently, -1 = none
  // Consecutive swap-in groups share a ring slot while they fit together (a "pack"): the small groups at the two
  // ends of the iteration would otherwise each hold a whole slot, and the link could run only a few small
  // transfers ahead of the compute stream.
  std::vector<int32_t> in_pack_of;                  // per swap-in group: its pack; pack p lives in slot p % n_slots
  std::vector<uint64_t> in_pack_off;                // per swap-in group: where it starts inside the slot
  std::vector<int32_t> in_pack_last_scatter;        // per pack, this iteration: swap-in batch scattered most recently, -1 = none
  std::vector<int32_t> in_slot_owner;               // per slot of the swap-in ring: pack whose bytes it holds, -1 = none
  std::vector<hipEvent_t> ev_fetched[2], ev_fetch_start[2];   // per group
  std::vector<uint8_t> in_group_state_drained;
  // SS_CFG_BARE_RING: sequence numbers of the ring transfers in place of their events (0 = none)
  std::vector<uint64_t> flush_seq;                  // per swap-out batch, this iteration: the transfer that carries it
  std::vector<uint64_t> group_last_flush_seq;       // per swap-out group: its latest transfer
  std::vector<uint64_t> fetch_seq;                  // per swap-in group: its transfer into the ring
  uint64_t last_flush_seq = 0;                      // the most recent transfer out of the ring
  int phase = 0;                                    // event set of the iteration being issued
  bool drained_once = false;                        // set `phase ^ 1` holds a completed iteration
  ss_desc_t *d_out = nullptr, *d_in = nullptr;    // device copies of the descriptors
  bool flat_next = false;                         // the batch being issued got its device addresses with the call
  uint32_t *d_out_chunk0 = nullptr, *d_in_chunk0 = nullptr;
  uint32_t *d_out_cdesc = nullptr, *d_in_cdesc = nullptr;
  size_t d_cap_out = 0, d_cap_in = 0, d_ccap_out = 0, d_ccap_in = 0;
  bool out_all_large = false;                     // every swap-out batch reaches engine_min_bytes_out (mean tensor size)
  int64_t last_engine_out = -1;                   // last swap-out batch of this iteration that went by copy engine
  std::vector<uint32_t> engine_in_issued;         // swap-in batches of this iteration that went by copy engine, in issue order
  std::vector<uint32_t> engine_out_issued;        // the same for swap-out
  bool loaded = false;
  // the action schedule of the last ss_apply_policy, for ss_dispatch: actions in schedule order and,
  // per operator, where its "before" and "after" runs start (act_start has 2 * n + 1 entries)
  std::vector<ss_action_t> actions;
  std::vector<uint32_t> act_start;
  bool have_actions = false;
};

struct ss_engine_queue;   // SS_CFG_BARE_RING: the thread that issues the ring transfers, and its state (ss_runtime.hip)

struct ss_ctx {
  ss_config_t cfg;
  int device = 0;
  // bound by the caller
  uint8_t *arena = nullptr;
  uint64_t arena_bytes = 0;
  hipStream_t compute = nullptr;
  bool bound = false;
  // owned
  uint8_t *staging = nullptr;       // pinned, host address
  uint8_t *staging_dev = nullptr;   // same memory, device address
  // swap streams: kernel batches of a direction take its streams in turn (cfg.out_streams / in_streams of
  // them), copy-engine batches always the first
  static constexpr int kMaxSwapStreams = 4;
  hipStream_t s_out[kMaxSwapStreams] = {}, s_in[kMaxSwapStreams] = {}, s_aux = nullptr;
  uint32_t n_s_out = 1, n_s_in = 1;
  hipStream_t s_flush = nullptr;    // copy-engine transfers out of the HBM ring
  bool pooled_streams = true;       // the swap streams go back to the process-wide pool at ss_destroy
  uint8_t *ring = nullptr;          // HBM ring of the staged swap-out path (cfg.ring_bytes, in slots of cfg.ring_slot_bytes)
  uint8_t *ring_in = nullptr;       // the same for the staged swap-in path
  uint32_t n_slots = 0;
  ss_engine_queue *eq = nullptr;    // SS_CFG_BARE_RING
  // SS_CFG_MEMORY_MARKERS: the compute stream's position as a running count in device memory
  uint64_t *d_mark = nullptr;       // device, 256 bytes; first word = count of the last marker the compute stream has passed
  uint64_t mark_count = 0;          // markers issued so far
  uint32_t *d_mark_gave_up = nullptr;                       // device: a wait for a marker ran into its limit
  uint32_t *h_mark_timeouts = nullptr, *d_mark_timeouts = nullptr;   // pinned word and its device address
  uint64_t mark_limit_ticks = 0;
  // SS_SYNC_ITERATION_END: end-of-iteration events of the swap streams, two sets used in turn (out streams 0..3,
  // in streams 4..7, ring-transfer stream 8); at most one iteration is outstanding behind the one being issued
  hipEvent_t ev_iter[2][9] = {};
  bool iter_pending[2] = {false, false};
  uint64_t iter_last_seq[2] = {0, 0};
  int iter_set = 0;
  std::vector<hipEvent_t> ev_ring;  // compute-stream markers, used round-robin
  size_t ev_next = 0;
  // trace
  ss_op_t *ops = nullptr;           // pinned
  ss_event_t *events = nullptr;     // pinned
  uint32_t n_ops = 0;
  uint64_t n_events = 0;
  int64_t balance = 0;
  std::unordered_map<std::string, uint32_t> tokens;
  std::unordered_map<std::string, uint32_t> stacks;
  // stage machine (Algo. 1)
  uint32_t stage = SS_STAGE_WARMUP, stable_step = 0;
  // scratch for scan / match (device + pinned mirrors), grown on demand
  void *d_scratch = nullptr;
  size_t d_scratch_bytes = 0;
  void *h_scratch = nullptr;        // pinned
  size_t h_scratch_bytes = 0;
  ss_sched sched;
  ss_stats_t stats;
};

// last failing HIP call of this thread: code, source file and line (ss_runtime.hip)
void ss_note_hip_error(int code, const char *file, int line);

#define SS_HIP(call)                                      \
  do {                                                    \
    hipError_t e__ = (call);                              \
    if (e__ != hipSuccess) {                              \
      ctx->stats.last_hip_error = (int32_t)e__;           \
      ss_note_hip_error((int)e__, __FILE__, __LINE__);    \
      (void)hipGetLastError();                            \
      return SS_E_HIP;                                    \
    }                                                     \
  } while (0)

static inline uint64_t ss_align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

// scratch management (ss_runtime.hip)
int ss_scratch_reserve(ss_ctx *ctx, size_t dev_bytes, size_t host_bytes);
// address of the static scratch array of ss_timeline_scan_static on the context's device (ss_scan.hip)
int ss_scan_static_init(ss_ctx *ctx);

// internal entry used by the greedy generator: timing + schedule without loading it
struct ss_applied {
  std::vector<ss_policy_item_t> resolved;
  std::vector<ss_action_t> actions;
  std::vector<ss_desc_t> out, in;
  std::vector<uint32_t> out_start, in_start, in_dep;
  std::vector<ss_event_t> pevents;
  uint64_t staging_bytes = 0, bytes_out = 0;
  uint32_t n_kept = 0, n_dropped = 0, n_late = 0;
};
int ss_apply_core(const ss_config_t &cfg, const ss_policy_item_t *policy, uint32_t k, const int32_t *new_idx,
                  const ss_tensor_t *tensors, uint32_t n_tensors, ss_applied &out);

// copy kernels (ss_copy.hip)
constexpr uint32_t SS_CHUNK_SHIFT = 16, SS_CHUNK_SHIFT_MIN = 12;
constexpr uint32_t SS_CHUNK_BYTES = 1u << SS_CHUNK_SHIFT;   // 64 KiB; small batches use down to 4 KiB
constexpr uint32_t SS_COPY_THREADS = 256;
void ss_launch_copy(hipStream_t s, uint32_t workgroups, uint32_t unroll, bool to_host, uint8_t *arena,
                    uint8_t *staging, const ss_desc_t *d_descs, const uint32_t *d_chunk0,
                    const uint32_t *d_chunk_desc, uint32_t n_chunks, uint32_t chunk_shift, uint32_t n_desc,
                    bool lds_lookup);
// one tensor by its two addresses, no descriptor table (16-byte aligned on both sides)
void ss_launch_copy_flat(hipStream_t s, uint32_t workgroups, const uint8_t *src, uint8_t *dst, uint64_t nbytes);
void ss_launch_fill(hipStream_t s, uint8_t *dst, uint64_t nbytes, uint8_t value);
// one thread that stores value at *flag once everything before it on stream s is complete (ss_mark_kernel)
void ss_launch_mark(hipStream_t s, uint64_t *flag, uint64_t value);
// one wave that holds stream s until *flag >= want (ss_wait_flag_kernel; bounded by limit_ticks of 10 ns)
void ss_launch_wait_flag(hipStream_t s, const uint64_t *flag, uint64_t want, uint64_t limit_ticks, uint32_t *gave_up,
                         uint32_t *timeouts);

// sequence aligner (ss_align.hip): ref_to_cur has n entries
int ss_align_core(ss_ctx *ctx, const ss_op_t *ref, uint32_t n, const ss_op_t *cur, uint32_t m,
                  int32_t *ref_to_cur, uint32_t *lcs, uint32_t *n_keys_out);
void ss_align_anchors(const ss_op_t *ref, uint32_t n, const ss_op_t *cur, const int32_t *ref_to_cur,
                      const ss_anchor_t *anchors, uint32_t k, int32_t *new_idx, uint8_t *level,
                      uint32_t *n_unmatched);
