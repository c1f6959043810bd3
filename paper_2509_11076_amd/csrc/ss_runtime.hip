// Host runtime of libss: context, streams and events, schedule loading, and the
// swap-out / swap-in / release calls with device-side ordering (Sec. 5.2 of the
// SmartSwap paper: swaps run on their own stream; a swapped-out block is handed
// back right after the operator that is running when the swap-out completes,
// by making the compute stream wait on the device instead of polling events on
// the host).
#include <algorithm>
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstring>
#include <deque>
#include <mutex>
#include <thread>

#include "ss_internal.h"

static thread_local int t_hip_code = 0, t_hip_line = 0;
static thread_local const char *t_hip_file = "";

void ss_note_hip_error(int code, const char *file, int line) {
  t_hip_code = code;
  t_hip_file = file;
  t_hip_line = line;
}

extern "C" int ss_last_hip_error(const char **name, const char **file, int *line) {
  if (name) *name = hipGetErrorName((hipError_t)t_hip_code);
  if (file) *file = t_hip_file;
  if (line) *line = t_hip_line;
  return t_hip_code;
}

extern "C" const char *ss_strerror(int code) {
  switch (code) {
    case SS_OK: return "ok";
    case SS_E_INVAL: return "invalid argument";
    case SS_E_NOMEM: return "out of memory (host, pinned or device) or staging too small";
    case SS_E_HIP: return "HIP call failed (see ss_stats_t.last_hip_error)";
    case SS_E_INFEASIBLE: return "no candidate left while memory still exceeds the budget";
    case SS_E_ORDER: return "events not in operator order";
    case SS_E_STATE: return "call out of sequence";
    case SS_E_CAPACITY: return "output array or configured capacity too small";
    case SS_E_TIMEOUT: return "a stream gave up waiting for a ring transfer";
    default: return "unknown error";
  }
}

extern "C" int ss_config_default(ss_config_t *cfg) {
  if (!cfg) return SS_E_INVAL;
  std::memset(cfg, 0, sizeof(*cfg));
  cfg->staging_bytes = 64ull << 20;
  cfg->link_bytes_per_op = 64ull << 20;
  cfg->engine_min_bytes = 4ull << 20;
  cfg->engine_min_bytes_out = 32ull << 20;
  cfg->align = 256;
  cfg->guard_bytes = 0;
  cfg->stage_m = 2;
  cfg->stage_n = 5;
  cfg->copy_path = SS_PATH_AUTO;
  cfg->copy_path_in = SS_PATH_AUTO;
  cfg->copy_workgroups = 0;
  cfg->max_ops = 65536;
  cfg->max_events = 1u << 20;
  cfg->flags = 0;
  return SS_OK;
}

static uint32_t default_workgroups() { return 64; }

// Ordering events only order work on this device (compute stream <-> swap streams); the host
// reads staging only after a stream synchronisation.  So they need no system-scope fence,
// which would write back and invalidate the L2 at every marker.
static unsigned fence_flag(const ss_config_t &cfg) {
  return (cfg.flags & SS_CFG_SYSTEM_FENCE) ? 0u : (unsigned)hipEventDisableSystemFence;
}

// Swap streams are kept for the life of the process and handed from a destroyed context to the next one that
// asks for the same role (device, direction, index): where the runtime places a new stream (its hardware queue,
// the copy engine its transfers go to) changes with every stream created, and with it how much a transfer costs
// the kernels that run beside it - a step of a PyTorch model measured at 34 ms took 42 ms in a later context of
// the same process, with nothing else changed.  With the streams kept, every context of a process runs where the
// first one did.
namespace {
struct pooled_stream { int device; int role; hipStream_t st; };
std::mutex g_pool_mu;
std::vector<pooled_stream> g_pool;      // streams not in use by a live context

hipError_t pool_take(int device, int role, hipStream_t *st) {
  {
    std::lock_guard<std::mutex> lock(g_pool_mu);
    for (size_t i = 0; i < g_pool.size(); ++i)
      if (g_pool[i].device == device && g_pool[i].role == role) {
        *st = g_pool[i].st;
        g_pool.erase(g_pool.begin() + (long)i);
        return hipSuccess;
      }
  }
  return hipStreamCreateWithFlags(st, hipStreamNonBlocking);      // default priority
}

void pool_give(int device, int role, hipStream_t st) {
  std::lock_guard<std::mutex> lock(g_pool_mu);
  g_pool.push_back({device, role, st});
}
constexpr int kRoleOut = 0, kRoleIn = 16, kRoleFlush = 32;
}  // namespace

// ---- SS_CFG_BARE_RING: the ring transfers, issued by a thread of the library's own -------------------
//
// What the dispatch thread would put before a transfer on its stream (waits for events) the thread does on the
// host: it takes the jobs in the order they were pushed, waits for each job's events (all recorded before the
// push), and only then enqueues the transfer, followed by a transfer of kFlagBytes whose first word is the job's
// sequence number, into the flag in device memory.  The stream thus carries copy-engine transfers and nothing
// else.  Sequence numbers grow by one per job for the life of the context; the stream runs its transfers in
// order, so "flag >= n" means that job n and every job before it are complete.  Every dependency of a job is on
// work issued before it was pushed, and none of that work waits for a later job, so the queue cannot block
// itself; a job whose events are late only holds back the jobs behind it.
struct ss_engine_job {
  hipEvent_t pre[3];
  int n_pre;
  void *dst;
  const void *src;
  size_t bytes;
  hipMemcpyKind kind;
  uint64_t seq;
  uint32_t dir, unit;            // what ss_batch_ms calls it: direction 2 or 3, ring group
};

struct ss_engine_queue {
  static constexpr size_t kFlagBytes = 65536;   // an 8-byte transfer is done by a kernel of the runtime, not by the copy engine
  static constexpr uint64_t kSources = 256;     // source buffers of the flag transfers, reused in turn
  int device = 0;
  hipStream_t stream = nullptr;                 // the context's stream for ring transfers
  uint64_t *d_flag = nullptr;                   // device memory, kFlagBytes; first word = last complete job
  uint8_t *h_src = nullptr;                     // pinned, kSources * kFlagBytes
  uint32_t *h_timeouts = nullptr, *d_timeouts = nullptr;   // a pinned word and its device address
  uint32_t *d_gave_up = nullptr;                // device memory: a wait ran into its limit; later waits do not poll
  uint64_t limit_ticks = 0;                     // bound of a wait, in ticks of 10 ns
  std::thread th;
  std::mutex mu;
  std::condition_variable cv, cv_idle;
  std::deque<ss_engine_job> q;
  bool stop = false, busy = false, started = false;
  uint64_t next_seq = 1;                        // dispatch thread
  uint64_t enqueued_seq = 0;                    // last job handed to the stream (under mu)
  uint64_t synced_seq = 0;                      // jobs up to here are known to be complete (the thread's own while it works; set by the drain while it idles)
  std::atomic<int> hip_error{0};                // first HIP error the thread met
  uint64_t waited_out = 0, waited_in = 0;       // dispatch thread: highest number a wait on the swap-out / swap-in stream covers
  // SS_CFG_TIMING: the transfers carry no events, so their times are taken on the host's clock.  A third
  // transfer behind each job copies the flag into pinned host memory, and a second thread, which makes no HIP
  // call at all, notes when it sees each number arrive.  A job starts when it is enqueued or when the job
  // before it is complete, whichever is later.
  bool timing = false;
  uint64_t *h_done = nullptr;                   // pinned, kFlagBytes; first word = last job seen complete by the host
  std::thread observer;
  std::atomic<bool> stop_observer{false};
  struct rec { uint64_t seq; uint32_t dir, unit; double t_enq, t_done; };
  std::vector<rec> recs;                        // the jobs of the iteration being issued (under mu)
  uint64_t observed = 0;                        // under mu
  std::vector<double> unit_start[2], unit_end[2];   // iteration drained last: per ring group, ms on the host's clock; < 0 = none
};

// Contexts that are still alive when the process ends (an exception on the caller's side, say) would leave
// their threads running while the runtime unmaps the pinned memory they look at.  This library's static objects
// are destroyed before those of the runtime it depends on, so the threads are stopped here: the watching thread
// always (it never blocks), the issuing thread if it is idle (else it is left to the process's end).
namespace {
std::mutex g_live_mu;
std::vector<ss_engine_queue *> g_live;
struct live_queues_reaper {
  ~live_queues_reaper() {
    std::lock_guard<std::mutex> lock(g_live_mu);
    for (ss_engine_queue *q : g_live) {
      if (q->timing && q->observer.joinable()) {
        q->stop_observer.store(true);
        q->observer.join();
      }
      bool idle;
      {
        std::lock_guard<std::mutex> lk(q->mu);
        idle = q->q.empty() && !q->busy;
        if (idle) q->stop = true;
      }
      if (!q->th.joinable()) continue;
      if (idle) {
        q->cv.notify_all();
        q->th.join();
      } else {
        q->th.detach();
      }
    }
    g_live.clear();
  }
} g_live_queues_reaper;
}  // namespace

static double host_ms() {
  return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

static void observer_thread(ss_engine_queue *q) {
  uint64_t last = 0;
  while (!q->stop_observer.load(std::memory_order_relaxed)) {
    const uint64_t v = *(volatile uint64_t *)q->h_done;
    if (v > last) {
      const double t = host_ms();
      std::lock_guard<std::mutex> lk(q->mu);
      for (auto &r : q->recs)
        if (r.seq > last && r.seq <= v) r.t_done = t;
      q->observed = last = v;
    } else {
      std::this_thread::yield();
    }
  }
}

static void engine_thread(ss_engine_queue *q) {
  auto note = [q](hipError_t e) {
    if (e == hipSuccess) return;
    int none = 0;
    q->hip_error.compare_exchange_strong(none, (int)e);
    (void)hipGetLastError();
  };
  note(hipSetDevice(q->device));
  for (;;) {
    ss_engine_job job;
    {
      std::unique_lock<std::mutex> lk(q->mu);
      q->cv.wait(lk, [q] { return q->stop || !q->q.empty(); });
      if (q->q.empty()) return;                 // asked to stop, nothing left
      job = q->q.front();
      q->q.pop_front();
      q->busy = true;
    }
    for (int i = 0; i < job.n_pre; ++i) note(hipEventSynchronize(job.pre[i]));
    if (job.seq > q->synced_seq + ss_engine_queue::kSources) {    // the source buffer's previous transfer may still be queued
      note(hipStreamSynchronize(q->stream));
      q->synced_seq = job.seq - 1;
    }
    uint64_t *src = (uint64_t *)(q->h_src + (size_t)(job.seq % ss_engine_queue::kSources) * ss_engine_queue::kFlagBytes);
    *src = job.seq;
    if (q->timing) {                            // noted before the transfer can complete: the watching thread looks it up
      std::lock_guard<std::mutex> lk(q->mu);
      q->recs.push_back({job.seq, job.dir, job.unit, host_ms(), -1.0});
    }
    if (job.bytes) note(hipMemcpyAsync(job.dst, job.src, job.bytes, job.kind, q->stream));
    // published even after a failure, so that nothing waits for this job in vain
    note(hipMemcpyAsync(q->d_flag, src, ss_engine_queue::kFlagBytes, hipMemcpyHostToDevice, q->stream));
    if (q->timing) note(hipMemcpyAsync(q->h_done, q->d_flag, ss_engine_queue::kFlagBytes, hipMemcpyDeviceToHost, q->stream));
    {
      std::lock_guard<std::mutex> lk(q->mu);
      q->enqueued_seq = job.seq;
      q->busy = false;
      if (q->q.empty()) q->cv_idle.notify_all();
    }
  }
}

static void eq_destroy(ss_ctx *ctx) {
  ss_engine_queue *q = ctx->eq;
  if (!q) return;
  {
    std::lock_guard<std::mutex> lock(g_live_mu);
    g_live.erase(std::remove(g_live.begin(), g_live.end(), q), g_live.end());
  }
  if (q->started) {
    {
      std::lock_guard<std::mutex> lk(q->mu);
      q->stop = true;
    }
    q->cv.notify_all();
    q->th.join();
    (void)hipStreamSynchronize(q->stream);
    if (q->timing) {
      q->stop_observer.store(true);
      q->observer.join();
    }
  }
  if (q->h_done) (void)hipHostFree(q->h_done);
  if (q->d_flag) (void)hipFree(q->d_flag);
  if (q->d_gave_up) (void)hipFree(q->d_gave_up);
  if (q->h_src) (void)hipHostFree(q->h_src);
  if (q->h_timeouts) (void)hipHostFree(q->h_timeouts);
  delete q;
  ctx->eq = nullptr;
}

static int eq_create(ss_ctx *ctx) {
  ss_engine_queue *q = new (std::nothrow) ss_engine_queue();
  if (!q) return SS_E_NOMEM;
  ctx->eq = q;
  q->device = ctx->device;
  q->stream = ctx->s_flush;
  q->limit_ticks = (uint64_t)(ctx->cfg.flag_wait_ms ? ctx->cfg.flag_wait_ms : 10000u) * 100000ull;
  if (hipMalloc((void **)&q->d_flag, ss_engine_queue::kFlagBytes) != hipSuccess ||
      hipMalloc((void **)&q->d_gave_up, 256) != hipSuccess ||
      hipHostMalloc((void **)&q->h_src, ss_engine_queue::kSources * ss_engine_queue::kFlagBytes, hipHostMallocDefault) != hipSuccess ||
      hipHostMalloc((void **)&q->h_timeouts, 64, hipHostMallocMapped) != hipSuccess) {
    (void)hipGetLastError();
    return SS_E_NOMEM;
  }
  std::memset(q->h_src, 0, ss_engine_queue::kSources * ss_engine_queue::kFlagBytes);
  std::memset(q->h_timeouts, 0, 64);
  SS_HIP(hipHostGetDevicePointer((void **)&q->d_timeouts, q->h_timeouts, 0));
  SS_HIP(hipMemcpy(q->d_flag, q->h_src, ss_engine_queue::kFlagBytes, hipMemcpyHostToDevice));
  SS_HIP(hipMemcpy(q->d_gave_up, q->h_timeouts + 4, 4, hipMemcpyHostToDevice));       // a word that stays zero
  if (ctx->cfg.flags & SS_CFG_TIMING) {
    if (hipHostMalloc((void **)&q->h_done, ss_engine_queue::kFlagBytes, hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      return SS_E_NOMEM;
    }
    std::memset(q->h_done, 0, ss_engine_queue::kFlagBytes);
    q->timing = true;
    q->observer = std::thread(observer_thread, q);
  }
  q->th = std::thread(engine_thread, q);
  q->started = true;
  {
    std::lock_guard<std::mutex> lock(g_live_mu);
    g_live.push_back(q);
  }
  return SS_OK;
}

// hands a transfer to the thread; returns its sequence number
static uint64_t eq_push(ss_ctx *ctx, void *dst, const void *src, size_t bytes, hipMemcpyKind kind,
                        const hipEvent_t *pre, int n_pre, uint32_t dir, uint32_t unit) {
  ss_engine_queue *q = ctx->eq;
  ss_engine_job job{};
  for (int i = 0; i < n_pre && i < 3; ++i) job.pre[i] = pre[i];
  job.n_pre = n_pre < 3 ? n_pre : 3;
  job.dst = dst;
  job.src = src;
  job.bytes = bytes;
  job.kind = kind;
  job.dir = dir;
  job.unit = unit;
  {
    std::lock_guard<std::mutex> lk(q->mu);
    job.seq = q->next_seq++;
    q->q.push_back(job);
  }
  q->cv.notify_one();
  return job.seq;
}

// every job pushed so far is on the stream
static void eq_wait_idle(ss_ctx *ctx) {
  ss_engine_queue *q = ctx->eq;
  if (!q || !q->started) return;
  std::unique_lock<std::mutex> lk(q->mu);
  q->cv_idle.wait(lk, [q] { return q->q.empty() && !q->busy; });
}

// job `seq` and every job before it have been handed to the stream
static void eq_wait_enqueued(ss_ctx *ctx, uint64_t seq) {
  ss_engine_queue *q = ctx->eq;
  if (!q || !q->started || seq == 0) return;
  std::unique_lock<std::mutex> lk(q->mu);
  while (q->enqueued_seq < seq) q->cv_idle.wait_for(lk, std::chrono::microseconds(100));
}

// stream st goes on only once job `seq` is complete (one wait per stream covers every earlier job)
static int eq_stream_wait(ss_ctx *ctx, hipStream_t st, uint64_t seq, uint64_t *covered) {
  if (seq == 0 || *covered >= seq) return SS_OK;
  ss_engine_queue *q = ctx->eq;
  ss_launch_wait_flag(st, q->d_flag, seq, q->limit_ticks, q->d_gave_up, q->d_timeouts);
  SS_HIP(hipGetLastError());
  *covered = seq;
  return SS_OK;
}

extern "C" int ss_create(ss_ctx **out, const ss_config_t *cfg_in) {
  return ss_guard([&]() -> int {
    if (!out) return SS_E_INVAL;
    *out = nullptr;
    ss_config_t cfg;
    ss_config_default(&cfg);
    if (cfg_in) cfg = *cfg_in;
    if (cfg.align < 16 || (cfg.align & (cfg.align - 1)) || cfg.guard_bytes % cfg.align ||
        cfg.link_bytes_per_op == 0 || cfg.max_ops == 0 || cfg.max_events == 0 ||
        cfg.max_ops > (1u << 23) || cfg.copy_path > SS_PATH_STAGED || cfg.copy_path_in > SS_PATH_STAGED)
      return SS_E_INVAL;
    if (cfg.ring_slot_bytes == 0) cfg.ring_slot_bytes = 256ull << 20;
    if (cfg.ring_bytes == 0) cfg.ring_bytes = 1024ull << 20;
    if (cfg.gather_workgroups == 0) cfg.gather_workgroups = 256;
    if (cfg.gather_workgroups > 4096 || cfg.ring_taper > 16 || cfg.copy_desc_lookup > 1) return SS_E_INVAL;
    if ((cfg.copy_path == SS_PATH_STAGED || cfg.copy_path_in == SS_PATH_STAGED) &&
        ((cfg.ring_slot_bytes & 255u) || cfg.ring_slot_bytes < 4096 || cfg.ring_bytes / cfg.ring_slot_bytes < 2 ||
         cfg.ring_bytes / cfg.ring_slot_bytes > 64))
      return SS_E_INVAL;
    if (cfg.copy_workgroups == 0) cfg.copy_workgroups = default_workgroups();
    if (cfg.copy_workgroups_out == 0) cfg.copy_workgroups_out = cfg.copy_workgroups;
    if (cfg.copy_unroll == 0) cfg.copy_unroll = 8;
    if (cfg.copy_workgroups > 4096 || cfg.copy_workgroups_out > 4096 || cfg.copy_unroll > 8) return SS_E_INVAL;
    if (cfg.flag_wait_ms > 600000u) return SS_E_INVAL;
    if (cfg.out_streams == 0) cfg.out_streams = 1;
    if (cfg.in_streams == 0) cfg.in_streams = 1;
    if (cfg.out_streams > ss_ctx::kMaxSwapStreams || cfg.in_streams > ss_ctx::kMaxSwapStreams) return SS_E_INVAL;

    ss_ctx *ctx = new (std::nothrow) ss_ctx();
    if (!ctx) return SS_E_NOMEM;
    ctx->cfg = cfg;
    std::memset(&ctx->stats, 0, sizeof(ctx->stats));
    int rc = SS_OK;
    auto fail_at = [&](int code, hipError_t e, int line) {
      ctx->stats.last_hip_error = (int32_t)e;
      ss_note_hip_error((int)e, __FILE__, line);
      (void)hipGetLastError();
      rc = code;
    };
#define fail(code, e) fail_at(code, e, __LINE__)
    hipError_t e;
    if ((e = hipGetDevice(&ctx->device)) != hipSuccess) fail(SS_E_HIP, e);
    if (rc == SS_OK) rc = ss_scan_static_init(ctx);
    if (rc == SS_OK && cfg.staging_bytes) {
      e = hipHostMalloc((void **)&ctx->staging, cfg.staging_bytes, hipHostMallocMapped | hipHostMallocPortable);
      if (e != hipSuccess) fail(SS_E_NOMEM, e);
      else if ((e = hipHostGetDevicePointer((void **)&ctx->staging_dev, ctx->staging, 0)) != hipSuccess)
        fail(SS_E_HIP, e);
    }
    if (rc == SS_OK && (e = hipHostMalloc((void **)&ctx->ops, (size_t)cfg.max_ops * sizeof(ss_op_t),
                                          hipHostMallocMapped)) != hipSuccess) fail(SS_E_NOMEM, e);
    if (rc == SS_OK && (e = hipHostMalloc((void **)&ctx->events, (size_t)cfg.max_events * sizeof(ss_event_t),
                                          hipHostMallocMapped)) != hipSuccess) fail(SS_E_NOMEM, e);
    // all streams at the default priority
    const bool any_staged = cfg.copy_path == SS_PATH_STAGED || cfg.copy_path_in == SS_PATH_STAGED;
    ctx->n_s_out = any_staged ? 1 : cfg.out_streams;
    ctx->n_s_in = any_staged ? 1 : cfg.in_streams;
    // With copy_cus > 0 the swap streams may place their kernels only on that many compute units (bit i of the
    // mask is compute unit i / n_xcd of die i % n_xcd on this part, so the first bits spread over the dies):
    // the copy kernel's long-lived waves then keep the compute stream's workgroups off those units only.
    // Streams with a unit mask are created non-blocking at the default priority like the others.
    std::vector<uint32_t> cu_mask;
    if (cfg.copy_cus) {
      hipDeviceProp_t prop;
      if ((e = hipGetDeviceProperties(&prop, ctx->device)) != hipSuccess) fail(SS_E_HIP, e);
      else {
        const uint32_t n_cu = (uint32_t)prop.multiProcessorCount;
        if (cfg.copy_cus > n_cu) rc = SS_E_INVAL;
        cu_mask.assign((n_cu + 31) / 32, 0u);
        for (uint32_t i = 0; i < cfg.copy_cus && rc == SS_OK; ++i) cu_mask[i / 32] |= 1u << (i % 32);
      }
    }
    ctx->pooled_streams = cu_mask.empty();          // streams with a unit mask are this context's own
    auto make_stream = [&](hipStream_t *st, int role) {
      if (cu_mask.empty()) return pool_take(ctx->device, role, st);
      return hipExtStreamCreateWithCUMask(st, (uint32_t)cu_mask.size(), cu_mask.data());
    };
    for (uint32_t i = 0; i < ctx->n_s_out && rc == SS_OK; ++i)
      if ((e = make_stream(&ctx->s_out[i], kRoleOut + (int)i)) != hipSuccess) fail(SS_E_HIP, e);
    for (uint32_t i = 0; i < ctx->n_s_in && rc == SS_OK; ++i)
      if ((e = make_stream(&ctx->s_in[i], kRoleIn + (int)i)) != hipSuccess) fail(SS_E_HIP, e);
    // The trace kernels (scan, match, align) run on the first swap-in stream: it is idle between iterations,
    // when they are called, and every further stream of the process has to share one of the few hardware
    // queues (4 per process here) with another - a stream that shares its queue with the stream of the
    // copy-engine transfers stands still for the length of every transfer.
    ctx->s_aux = ctx->s_in[0];
    if (rc == SS_OK && (cfg.copy_path == SS_PATH_STAGED || cfg.copy_path_in == SS_PATH_STAGED)) {
      // gathers / scatters and direct batches of a direction share that direction's one stream; the copy-engine
      // transfers out of and into the rings share a third
      ctx->n_slots = (uint32_t)(cfg.ring_bytes / cfg.ring_slot_bytes);
      if ((e = pool_take(ctx->device, kRoleFlush, &ctx->s_flush)) != hipSuccess) fail(SS_E_HIP, e);
      if (rc == SS_OK && cfg.copy_path == SS_PATH_STAGED &&
          (e = hipMalloc((void **)&ctx->ring, (size_t)ctx->n_slots * cfg.ring_slot_bytes)) != hipSuccess)
        fail(SS_E_NOMEM, e);
      if (rc == SS_OK && cfg.copy_path_in == SS_PATH_STAGED &&
          (e = hipMalloc((void **)&ctx->ring_in, (size_t)ctx->n_slots * cfg.ring_slot_bytes)) != hipSuccess)
        fail(SS_E_NOMEM, e);
      if (rc == SS_OK && (cfg.flags & SS_CFG_BARE_RING)) rc = eq_create(ctx);
    }
    if (rc == SS_OK && (cfg.flags & SS_CFG_MEMORY_MARKERS)) {
      ctx->mark_limit_ticks = (uint64_t)(cfg.flag_wait_ms ? cfg.flag_wait_ms : 10000u) * 100000ull;
      if ((e = hipMalloc((void **)&ctx->d_mark, 256)) != hipSuccess) fail(SS_E_NOMEM, e);
      else if ((e = hipMalloc((void **)&ctx->d_mark_gave_up, 256)) != hipSuccess) fail(SS_E_NOMEM, e);
      else if ((e = hipHostMalloc((void **)&ctx->h_mark_timeouts, 256, hipHostMallocMapped)) != hipSuccess) fail(SS_E_NOMEM, e);
      else {
        std::memset(ctx->h_mark_timeouts, 0, 256);
        if ((e = hipHostGetDevicePointer((void **)&ctx->d_mark_timeouts, ctx->h_mark_timeouts, 0)) != hipSuccess) fail(SS_E_HIP, e);
        else if ((e = hipMemcpy(ctx->d_mark, ctx->h_mark_timeouts, 256, hipMemcpyHostToDevice)) != hipSuccess) fail(SS_E_HIP, e);
        else if ((e = hipMemcpy(ctx->d_mark_gave_up, ctx->h_mark_timeouts, 256, hipMemcpyHostToDevice)) != hipSuccess) fail(SS_E_HIP, e);
      }
    }
    for (int i = 0; i < 2048 && rc == SS_OK; ++i) {
      hipEvent_t ev;
      if ((e = hipEventCreateWithFlags(&ev, hipEventDisableTiming | fence_flag(cfg))) != hipSuccess) fail(SS_E_HIP, e);
      else ctx->ev_ring.push_back(ev);
    }
#undef fail
    if (rc != SS_OK) {
      ss_destroy(ctx);
      return rc;
    }
    *out = ctx;
    return SS_OK;
  });
}

static void free_events(std::vector<hipEvent_t> &v) {
  for (hipEvent_t e : v)
    if (e) (void)hipEventDestroy(e);
  v.clear();
}

// host joins every swap stream of both directions
static int sync_swap_streams(ss_ctx *ctx) {
  eq_wait_idle(ctx);                  // the ring transfers pushed so far are on their stream
  for (uint32_t i = 0; i < ctx->n_s_out; ++i)
    if (ctx->s_out[i]) SS_HIP(hipStreamSynchronize(ctx->s_out[i]));
  for (uint32_t i = 0; i < ctx->n_s_in; ++i)
    if (ctx->s_in[i]) SS_HIP(hipStreamSynchronize(ctx->s_in[i]));
  if (ctx->s_flush) SS_HIP(hipStreamSynchronize(ctx->s_flush));
  return SS_OK;
}

static void sched_release(ss_sched &s) {
  for (int p = 0; p < 2; ++p) {
    free_events(s.ev_out_done[p]);
    free_events(s.ev_in_done[p]);
    free_events(s.ev_out_start[p]);
    free_events(s.ev_in_start[p]);
    free_events(s.ev_gathered[p]);
    free_events(s.ev_flush_start[p]);
    free_events(s.ev_fetched[p]);
    free_events(s.ev_fetch_start[p]);
  }
  free_events(s.ev_free_at);
  free_events(s.ev_wait_at);
  if (s.d_out) (void)hipFree(s.d_out);
  if (s.d_in) (void)hipFree(s.d_in);
  if (s.d_out_chunk0) (void)hipFree(s.d_out_chunk0);
  if (s.d_in_chunk0) (void)hipFree(s.d_in_chunk0);
  if (s.d_out_cdesc) (void)hipFree(s.d_out_cdesc);
  if (s.d_in_cdesc) (void)hipFree(s.d_in_cdesc);
  s.d_out_cdesc = s.d_in_cdesc = nullptr;
  s.d_ccap_out = s.d_ccap_in = 0;
  s.d_out = s.d_in = nullptr;
  s.d_out_chunk0 = s.d_in_chunk0 = nullptr;
  s.d_cap_out = s.d_cap_in = 0;
  s.loaded = false;
}

extern "C" int ss_destroy(ss_ctx *ctx) {
  if (!ctx) return SS_E_INVAL;
  (void)sync_swap_streams(ctx);
  eq_destroy(ctx);
  sched_release(ctx->sched);
  for (hipEvent_t ev : ctx->ev_ring) (void)hipEventDestroy(ev);
  for (int p = 0; p < 2; ++p)
    for (int k = 0; k < 9; ++k)
      if (ctx->ev_iter[p][k]) (void)hipEventDestroy(ctx->ev_iter[p][k]);
  for (int i = 0; i < ss_ctx::kMaxSwapStreams; ++i) {       // joined above: nothing is pending on them
    if (ctx->s_out[i]) ctx->pooled_streams ? pool_give(ctx->device, kRoleOut + i, ctx->s_out[i]) : (void)hipStreamDestroy(ctx->s_out[i]);
    if (ctx->s_in[i]) ctx->pooled_streams ? pool_give(ctx->device, kRoleIn + i, ctx->s_in[i]) : (void)hipStreamDestroy(ctx->s_in[i]);
  }
  if (ctx->s_flush) pool_give(ctx->device, kRoleFlush, ctx->s_flush);
  if (ctx->d_mark) (void)hipFree(ctx->d_mark);
  if (ctx->d_mark_gave_up) (void)hipFree(ctx->d_mark_gave_up);
  if (ctx->h_mark_timeouts) (void)hipHostFree(ctx->h_mark_timeouts);
  if (ctx->ring) (void)hipFree(ctx->ring);
  if (ctx->ring_in) (void)hipFree(ctx->ring_in);
  if (ctx->staging) (void)hipHostFree(ctx->staging);
  if (ctx->ops) (void)hipHostFree(ctx->ops);
  if (ctx->events) (void)hipHostFree(ctx->events);
  if (ctx->d_scratch) (void)hipFree(ctx->d_scratch);
  if (ctx->h_scratch) (void)hipHostFree(ctx->h_scratch);
  delete ctx;
  return SS_OK;
}

extern "C" int ss_bind(ss_ctx *ctx, void *arena, uint64_t arena_bytes, void *compute_stream) {
  // arena == NULL with arena_bytes == 0: no arena; every tensor's device address is given when its batch is
  // issued (ss_swap_out_from / ss_swap_in_to)
  if (!ctx || (!arena && arena_bytes) || ((uintptr_t)arena & 15u)) return SS_E_INVAL;
  ctx->arena = (uint8_t *)arena;
  ctx->arena_bytes = arena_bytes;
  ctx->compute = (hipStream_t)compute_stream;
  ctx->bound = true;
  ctx->sched.loaded = false;     // descriptors were validated against the previous arena
  return SS_OK;
}

int ss_scratch_reserve(ss_ctx *ctx, size_t dev_bytes, size_t host_bytes) {
  if (dev_bytes > ctx->d_scratch_bytes) {
    if (ctx->d_scratch) SS_HIP(hipFree(ctx->d_scratch));
    ctx->d_scratch = nullptr;
    ctx->d_scratch_bytes = 0;
    size_t want = ss_align_up(dev_bytes + dev_bytes / 4, 1 << 20);
    hipError_t e = hipMalloc(&ctx->d_scratch, want);
    if (e != hipSuccess) {
      ctx->stats.last_hip_error = (int32_t)e;
      ss_note_hip_error((int)e, __FILE__, __LINE__);
      (void)hipGetLastError();
      return SS_E_NOMEM;
    }
    ctx->d_scratch_bytes = want;
  }
  if (host_bytes > ctx->h_scratch_bytes) {
    if (ctx->h_scratch) SS_HIP(hipHostFree(ctx->h_scratch));
    ctx->h_scratch = nullptr;
    ctx->h_scratch_bytes = 0;
    size_t want = ss_align_up(host_bytes + host_bytes / 4, 1 << 20);
    hipError_t e = hipHostMalloc(&ctx->h_scratch, want, hipHostMallocDefault);
    if (e != hipSuccess) {
      ctx->stats.last_hip_error = (int32_t)e;
      ss_note_hip_error((int)e, __FILE__, __LINE__);
      (void)hipGetLastError();
      return SS_E_NOMEM;
    }
    ctx->h_scratch_bytes = want;
  }
  return SS_OK;
}

// ---- schedule ------------------------------------------------------------------

// per-iteration state of the staged swap-out path
static void ring_reset(ss_sched &s, uint32_t n_slots) {
  std::fill(s.done_ev_of.begin(), s.done_ev_of.end(), -1);
  std::fill(s.ring_state.begin(), s.ring_state.end(), 0);
  for (size_t g = 0; g < s.groups.size(); ++g) {
    s.group_pending[g] = s.groups[g].last - s.groups[g].first + 1;
    s.group_gathered[g] = s.group_started[g] = 0;
    s.group_last_flush[g] = -1;
  }
  s.slot_owner.assign(n_slots, -1);
  s.in_slot_owner.assign(n_slots, -1);
  std::fill(s.in_group_state.begin(), s.in_group_state.end(), 0);
  std::fill(s.in_group_last_scatter.begin(), s.in_group_last_scatter.end(), -1);
  std::fill(s.in_pack_last_scatter.begin(), s.in_pack_last_scatter.end(), -1);
  std::fill(s.out_staged.begin(), s.out_staged.end(), 0);
  s.last_flush_batch = s.last_gather_batch = s.last_direct_out = s.max_out_issued = -1;
  s.out_of_order = false;
  for (int64_t &x : s.last_out_on) x = -1;
  std::fill(s.flush_seq.begin(), s.flush_seq.end(), 0);
  std::fill(s.group_last_flush_seq.begin(), s.group_last_flush_seq.end(), 0);
  std::fill(s.fetch_seq.begin(), s.fetch_seq.end(), 0);
  s.last_flush_seq = 0;
  s.engine_in_issued.clear();
  s.engine_out_issued.clear();
}

static int check_descs(const ss_ctx *ctx, const ss_desc_t *d, uint32_t n) {
  const bool no_arena = ctx->arena == nullptr;        // addresses come with the batches: nothing to check them against
  for (uint32_t i = 0; i < n; ++i) {
    if ((d[i].dev_off & 15u) || (d[i].host_off & 15u)) return SS_E_INVAL;
    if (!no_arena && (d[i].dev_off > ctx->arena_bytes || d[i].nbytes > ctx->arena_bytes - d[i].dev_off)) return SS_E_INVAL;
    if (d[i].host_off > ctx->cfg.staging_bytes || d[i].nbytes > ctx->cfg.staging_bytes - d[i].host_off)
      return SS_E_NOMEM;
    if (d[i].nbytes > (1ull << 40)) return SS_E_INVAL;
  }
  return SS_OK;
}

static int check_batches(const uint32_t *start, uint32_t nb, uint32_t n) {
  if (nb == 0) return n == 0 ? SS_OK : SS_E_INVAL;
  if (!start || start[0] != 0 || start[nb] != n) return SS_E_INVAL;
  for (uint32_t b = 0; b < nb; ++b)
    if (start[b + 1] < start[b]) return SS_E_INVAL;
  return SS_OK;
}

static int ensure_events(ss_ctx *ctx, std::vector<hipEvent_t> &v, size_t n, unsigned flags) {
  while (v.size() < n) {
    hipEvent_t e;
    SS_HIP(hipEventCreateWithFlags(&e, flags));
    v.push_back(e);
  }
  return SS_OK;
}

// chunk-prefix per descriptor, restarting at every batch; entry [start[b+1]] of a
// batch's run is read as its sentinel, so each batch gets count + 1 entries.
// cdesc lists, batch after batch, the descriptor (counted from the batch's first) of every chunk;
// cbase[b] is where batch b's chunks start in it.
// A batch is cut into 64 KiB chunks unless that gives fewer than 256 of them (four per workgroup of
// the default grid): then the chunk size is halved down to 4 KiB, so that a batch of a few small
// tensors still spreads over the grid instead of running on two or three workgroups.
static void build_chunks(const std::vector<ss_desc_t> &d, const std::vector<uint32_t> &start,
                         std::vector<uint32_t> &chunk0, std::vector<uint32_t> &cdesc,
                         std::vector<uint64_t> &cbase, std::vector<uint8_t> &shift) {
  size_t nb = start.size() ? start.size() - 1 : 0;
  chunk0.assign(d.size() + nb, 0);
  cdesc.clear();
  cbase.assign(nb + 1, 0);
  shift.assign(nb, (uint8_t)SS_CHUNK_SHIFT);
  for (size_t b = 0; b < nb; ++b) {
    uint32_t sh = SS_CHUNK_SHIFT;
    for (; sh > SS_CHUNK_SHIFT_MIN; --sh) {
      uint64_t total = 0;
      for (uint32_t i = start[b]; i < start[b + 1]; ++i) total += (d[i].nbytes + (1ull << sh) - 1) >> sh;
      if (total >= 256) break;
    }
    shift[b] = (uint8_t)sh;
    uint32_t run = 0;
    size_t base = start[b] + b;
    cbase[b] = cdesc.size();
    for (uint32_t i = start[b]; i < start[b + 1]; ++i) {
      chunk0[base + (i - start[b])] = run;
      const uint32_t n = (uint32_t)((d[i].nbytes + (1ull << sh) - 1) >> sh);
      cdesc.insert(cdesc.end(), n, i - start[b]);
      run += n;
    }
    chunk0[base + (start[b + 1] - start[b])] = run;
  }
  cbase[nb] = cdesc.size();
}

extern "C" int ss_load_schedule(ss_ctx *ctx, const ss_desc_t *descs_out, uint32_t n_out,
                                const uint32_t *out_start, uint32_t n_out_batches,
                                const ss_desc_t *descs_in, uint32_t n_in, const uint32_t *in_start,
                                uint32_t n_in_batches, const uint32_t *in_dep) {
  return ss_guard([&]() -> int {
    if (!ctx || (n_out && !descs_out) || (n_in && !descs_in)) return SS_E_INVAL;
    if (!ctx->bound) return SS_E_STATE;
    int rc;
    if ((rc = check_batches(out_start, n_out_batches, n_out)) != SS_OK) return rc;
    if ((rc = check_batches(in_start, n_in_batches, n_in)) != SS_OK) return rc;
    for (uint32_t b = 0; in_dep && b < n_in_batches; ++b)
      if (n_out_batches == 0 || in_dep[b] >= n_out_batches) return SS_E_INVAL;
    ss_sched &s = ctx->sched;
    s.have_actions = false;       // a schedule loaded here carries no actions; ss_apply_policy adds them
    // the same schedule as the one already loaded (a fixed operator sequence in the Stable stage): it was
    // validated against this arena and staging area when it was loaded; device tables, chunk tables and
    // events stay, only the per-iteration state starts over
    {
      std::vector<uint32_t> dep(n_in_batches);
      for (uint32_t b = 0; b < n_in_batches; ++b) dep[b] = in_dep ? in_dep[b] : (n_out_batches ? n_out_batches - 1 : 0);
      const bool same =
          s.loaded && s.out.size() == n_out && s.in.size() == n_in && s.out_start.size() == (size_t)n_out_batches + 1 &&
          s.in_start.size() == (size_t)n_in_batches + 1 && s.in_dep == dep &&
          (n_out == 0 || std::memcmp(s.out.data(), descs_out, (size_t)n_out * sizeof(ss_desc_t)) == 0) &&
          (n_in == 0 || std::memcmp(s.in.data(), descs_in, (size_t)n_in * sizeof(ss_desc_t)) == 0) &&
          (n_out_batches == 0 || std::memcmp(s.out_start.data(), out_start, ((size_t)n_out_batches + 1) * 4) == 0) &&
          (n_in_batches == 0 || std::memcmp(s.in_start.data(), in_start, ((size_t)n_in_batches + 1) * 4) == 0);
      if (same) {
        // nothing of the previous iteration may still be in flight
        if ((rc = sync_swap_streams(ctx)) != SS_OK) return rc;
        std::fill(s.out_waited.begin(), s.out_waited.end(), 0);
        std::fill(s.out_issued.begin(), s.out_issued.end(), 0);
        std::fill(s.in_waited.begin(), s.in_waited.end(), 0);
        std::fill(s.in_issued.begin(), s.in_issued.end(), 0);
        s.last_engine_out = -1;
        ring_reset(s, ctx->n_slots);
        return SS_OK;
      }
    }
    if ((rc = check_descs(ctx, descs_out, n_out)) != SS_OK) return rc;
    if ((rc = check_descs(ctx, descs_in, n_in)) != SS_OK) return rc;
    // staging slots of the swap-out side must be pairwise disjoint
    {
      std::vector<std::pair<uint64_t, uint64_t>> iv;
      iv.reserve(n_out);
      for (uint32_t i = 0; i < n_out; ++i)
        if (descs_out[i].nbytes) iv.emplace_back(descs_out[i].host_off, descs_out[i].host_off + descs_out[i].nbytes);
      std::sort(iv.begin(), iv.end());
      for (size_t i = 1; i < iv.size(); ++i)
        if (iv[i].first < iv[i - 1].second) return SS_E_INVAL;
    }
    // nothing of the previous schedule may still be in flight
    if ((rc = sync_swap_streams(ctx)) != SS_OK) return rc;
    s.drained_once = false;      // the other event set belongs to the schedule that is being replaced

    s.loaded = false;
    s.out.assign(descs_out, descs_out + n_out);
    s.in.assign(descs_in, descs_in + n_in);
    s.out_start.assign(out_start ? out_start : nullptr, out_start ? out_start + n_out_batches + 1 : nullptr);
    s.in_start.assign(in_start ? in_start : nullptr, in_start ? in_start + n_in_batches + 1 : nullptr);
    if (s.out_start.empty()) s.out_start.push_back(0);
    if (s.in_start.empty()) s.in_start.push_back(0);
    s.in_dep.resize(n_in_batches);
    for (uint32_t b = 0; b < n_in_batches; ++b) s.in_dep[b] = in_dep ? in_dep[b] : (n_out_batches ? n_out_batches - 1 : 0);
    build_chunks(s.out, s.out_start, s.out_chunk0, s.out_cdesc, s.out_cbase, s.out_shift);
    build_chunks(s.in, s.in_start, s.in_chunk0, s.in_cdesc, s.in_cbase, s.in_shift);
    s.out_of_tensor.clear();
    s.in_of_tensor.clear();
    s.out_batch_of.assign(n_out, 0);
    s.in_batch_of.assign(n_in, 0);
    for (uint32_t b = 0; b < n_out_batches; ++b)
      for (uint32_t i = s.out_start[b]; i < s.out_start[b + 1]; ++i) {
        s.out_batch_of[i] = b;
        s.out_of_tensor[s.out[i].tensor_id] = i;
      }
    for (uint32_t b = 0; b < n_in_batches; ++b)
      for (uint32_t i = s.in_start[b]; i < s.in_start[b + 1]; ++i) {
        s.in_batch_of[i] = b;
        s.in_of_tensor[s.in[i].tensor_id] = i;
      }
    s.out_waited.assign(n_out_batches, 0);
    s.out_issued.assign(n_out_batches, 0);
    s.in_waited.assign(n_in_batches, 0);
    s.in_issued.assign(n_in_batches, 0);
    s.last_engine_out = -1;
    // staged swap-out: group consecutive batches whose staging slots form one gap-free range (every size
    // a multiple of the slot alignment, no guards) of at most one ring slot
    s.groups.clear();
    s.group_bytes.clear();
    s.group_of.assign(n_out_batches, -1);
    // Group sizes are tapered at the two ends of the iteration where the link would otherwise wait for a
    // full slot: the first swap-out groups double from kTaperMin up to a slot (a group leaves only once it is
    // complete, so the link starts after the first small group instead of after a slot's worth of forward
    // pass), the first swap-in groups double likewise (the backward pass goes on as soon as the first small
    // group is back instead of after a whole slot), and the last swap-in groups shrink down to kTaperMin, each
    // at most 1/n of what is still to come (what the backward pass still has to compute once the last byte is
    // back shrinks with the last group; n = 2 halves them, which is right when the operators that use a group
    // take far less time than the link needs for the next one; when they take a fraction r of it, a group
    // must not be smaller than r times the one before, or the compute stream falls behind while the small
    // groups arrive and catches up only after the last one: n >= 1 / (1 - r)).  kTaperMin is an eighth of a slot.
    const uint64_t kTaperMin = std::max<uint64_t>(ctx->cfg.ring_slot_bytes / 8, 256);
    const bool taper_in = ctx->cfg.ring_taper != 1, taper_out = taper_in;
    const uint64_t taper_den = ctx->cfg.ring_taper >= 2 ? ctx->cfg.ring_taper : 2;
    if (ctx->cfg.copy_path == SS_PATH_STAGED && ctx->ring) {
      const uint64_t slot_full = ctx->cfg.ring_slot_bytes;
      uint64_t grouped = 0;                       // bytes in the groups closed so far
      uint64_t slot = taper_out ? std::min(slot_full, kTaperMin) : slot_full;
      bool open = false;
      for (uint32_t b = 0; b < n_out_batches; ++b) {
        const uint32_t lo = s.out_start[b], hi = s.out_start[b + 1];
        bool ok = hi > lo && ctx->cfg.guard_bytes == 0;
        uint64_t total = 0;
        for (uint32_t i = lo; i < hi && ok; ++i) {
          ok = s.out[i].nbytes != 0 && s.out[i].nbytes % ctx->cfg.align == 0 &&
               (i == lo || s.out[i].host_off == s.out[i - 1].host_off + s.out[i - 1].nbytes);
          total += s.out[i].nbytes;
        }
        ok = ok && total <= slot_full;
        if (!ok) { open = false; continue; }
        if (open) {
          ss_sched::out_group &g = s.groups.back();
          if (s.out[lo].host_off == g.host_lo + g.bytes && g.bytes + total <= slot) {
            g.last = b;
            g.bytes += total;
            s.group_of[b] = (int32_t)s.groups.size() - 1;
            continue;
          }
          grouped += g.bytes;
          if (taper_out) slot = std::min(slot_full, std::max(kTaperMin, grouped));
        }
        s.groups.push_back(ss_sched::out_group{b, b, s.out[lo].host_off, total});
        s.group_of[b] = (int32_t)s.groups.size() - 1;
        open = true;
      }
      for (const ss_sched::out_group &g : s.groups) s.group_bytes.push_back(g.bytes);
    }
    // staged swap-in: consecutive batches whose staging slots together form one gap-free range (slots are
    // pairwise disjoint, so: the range they span is as long as their sizes add up to) of at most one ring slot
    s.in_groups.clear();
    s.in_group_bytes.clear();
    s.in_group_outs.clear();
    s.in_group_of.assign(n_in_batches, -1);
    if (ctx->cfg.copy_path_in == SS_PATH_STAGED && ctx->ring_in && ctx->cfg.guard_bytes == 0) {
      const uint64_t slot_full = ctx->cfg.ring_slot_bytes;
      uint64_t in_grouped = 0;                    // bytes in the groups made so far
      uint64_t remaining = 0;                     // bytes of the batches from f on
      for (uint32_t i = 0; i < n_in; ++i) remaining += s.in[i].nbytes;
      for (uint32_t f = 0; f < n_in_batches;) {
        const uint64_t slot = taper_in ? std::min(slot_full, std::min(std::max(kTaperMin, remaining / taper_den),
                                                                      std::max(kTaperMin, in_grouped))) : slot_full;
        uint64_t lo_off = ~0ull, hi_off = 0, total = 0;
        int64_t best = -1;
        uint64_t best_lo = 0, best_total = 0;
        for (uint32_t e = f; e < n_in_batches; ++e) {
          bool ok = s.in_start[e + 1] > s.in_start[e];
          for (uint32_t i = s.in_start[e]; i < s.in_start[e + 1] && ok; ++i) {
            ok = s.in[i].nbytes != 0 && s.in[i].nbytes % ctx->cfg.align == 0;
            lo_off = std::min(lo_off, s.in[i].host_off);
            hi_off = std::max(hi_off, s.in[i].host_off + s.in[i].nbytes);
            total += s.in[i].nbytes;
          }
          if (!ok || total > (e == f ? slot_full : slot)) break;      // a single batch may fill a whole slot
          if (hi_off - lo_off == total) { best = e; best_lo = lo_off; best_total = total; }
        }
        if (best < 0) {
          for (uint32_t i = s.in_start[f]; i < s.in_start[f + 1]; ++i) remaining -= s.in[i].nbytes;
          ++f;
          continue;
        }
        remaining -= best_total;
        in_grouped += best_total;
        const int32_t g = (int32_t)s.in_groups.size();
        s.in_groups.push_back(ss_sched::in_group{f, (uint32_t)best, best_lo, best_total});
        s.in_group_bytes.push_back(best_total);
        std::vector<uint32_t> outs;
        for (uint32_t b = f; b <= (uint32_t)best; ++b) {
          s.in_group_of[b] = g;
          for (uint32_t i = s.in_start[b]; i < s.in_start[b + 1]; ++i) {
            auto it = s.out_of_tensor.find(s.in[i].tensor_id);
            if (it != s.out_of_tensor.end()) outs.push_back(s.out_batch_of[it->second]);
            else outs.push_back(s.in_dep[b]);
          }
        }
        std::sort(outs.begin(), outs.end());
        outs.erase(std::unique(outs.begin(), outs.end()), outs.end());
        s.in_group_outs.push_back(std::move(outs));
        f = (uint32_t)best + 1;
      }
      // packs: consecutive groups share a slot while they fit together
      s.in_pack_of.assign(s.in_groups.size(), 0);
      s.in_pack_off.assign(s.in_groups.size(), 0);
      int32_t pack = -1;
      uint64_t used = slot_full;
      for (size_t g = 0; g < s.in_groups.size(); ++g) {
        const uint64_t need = ss_align_up(s.in_groups[g].bytes, 256);
        if (used + need > slot_full) {
          ++pack;
          used = 0;
        }
        s.in_pack_of[g] = pack;
        s.in_pack_off[g] = used;
        used += need;
      }
      s.in_pack_last_scatter.assign((size_t)(pack + 1), -1);
    } else {
      s.in_pack_of.clear();
      s.in_pack_off.clear();
      s.in_pack_last_scatter.clear();
    }
    s.in_group_state.assign(s.in_groups.size(), 0);
    s.in_group_state_drained.assign(s.in_groups.size(), 0);
    s.in_group_last_scatter.assign(s.in_groups.size(), -1);
    // SS_PATH_AUTO (and the batches SS_PATH_STAGED leaves alone): one path for the whole swap-out side
    s.out_all_large = ctx->cfg.engine_min_bytes_out != 0 && n_out_batches != 0;
    for (uint32_t b = 0; b < n_out_batches && s.out_all_large; ++b) {
      if (s.group_of[b] >= 0) continue;
      uint64_t total = 0;
      const uint32_t cnt = s.out_start[b + 1] - s.out_start[b];
      for (uint32_t i = s.out_start[b]; i < s.out_start[b + 1]; ++i) total += s.out[i].nbytes;
      if (cnt && total / cnt < ctx->cfg.engine_min_bytes_out) s.out_all_large = false;
    }
    s.done_ev_of.assign(n_out_batches, -1);
    s.done_ev_of_drained.assign(n_out_batches, -1);
    s.out_staged.assign(n_out_batches, 0);
    s.ring_state.assign(n_out_batches, 0);
    s.group_pending.assign(s.groups.size(), 0);
    s.group_gathered.assign(s.groups.size(), 0);
    s.group_started.assign(s.groups.size(), 0);
    s.group_last_flush.assign(s.groups.size(), -1);
    s.flush_seq.assign(n_out_batches, 0);
    s.group_last_flush_seq.assign(s.groups.size(), 0);
    s.fetch_seq.assign(s.in_groups.size(), 0);
    ring_reset(s, ctx->n_slots);

    const bool stall = (ctx->cfg.flags & SS_CFG_STALL_TIMING) != 0;
    const unsigned evflags = ((ctx->cfg.flags & (SS_CFG_TIMING | SS_CFG_STALL_TIMING)) ? hipEventDefault
                                                                                       : hipEventDisableTiming) |
                             fence_flag(ctx->cfg);
    if (stall) {
      if ((rc = ensure_events(ctx, s.ev_free_at, n_out_batches, evflags)) != SS_OK) return rc;
      if ((rc = ensure_events(ctx, s.ev_wait_at, n_in_batches, evflags)) != SS_OK) return rc;
    }
    for (int p = 0; p < 2; ++p) {
      if ((rc = ensure_events(ctx, s.ev_out_done[p], n_out_batches, evflags)) != SS_OK) return rc;
      if (!s.groups.empty()) {
        if ((rc = ensure_events(ctx, s.ev_gathered[p], n_out_batches, evflags)) != SS_OK) return rc;
        if ((ctx->cfg.flags & SS_CFG_TIMING) &&
            (rc = ensure_events(ctx, s.ev_flush_start[p], s.groups.size(), evflags)) != SS_OK) return rc;
      }
      if (!s.in_groups.empty()) {
        if ((rc = ensure_events(ctx, s.ev_fetched[p], s.in_groups.size(), evflags)) != SS_OK) return rc;
        if ((ctx->cfg.flags & SS_CFG_TIMING) &&
            (rc = ensure_events(ctx, s.ev_fetch_start[p], s.in_groups.size(), evflags)) != SS_OK) return rc;
      }
      if ((rc = ensure_events(ctx, s.ev_in_done[p], n_in_batches, evflags)) != SS_OK) return rc;
      if (ctx->cfg.flags & SS_CFG_TIMING) {
        if ((rc = ensure_events(ctx, s.ev_out_start[p], n_out_batches, evflags)) != SS_OK) return rc;
        if ((rc = ensure_events(ctx, s.ev_in_start[p], n_in_batches, evflags)) != SS_OK) return rc;
      }
    }
    // device copies of descriptors and chunk tables
    auto upload = [&](const std::vector<ss_desc_t> &d, const std::vector<uint32_t> &c, ss_desc_t *&dd,
                      uint32_t *&dc, size_t &cap) -> int {
      if (d.empty()) return SS_OK;
      if (d.size() > cap) {
        if (dd) SS_HIP(hipFree(dd));
        if (dc) SS_HIP(hipFree(dc));
        dd = nullptr; dc = nullptr; cap = 0;
        size_t want = d.size() + d.size() / 2 + 64;
        hipError_t e = hipMalloc((void **)&dd, want * sizeof(ss_desc_t));
        if (e == hipSuccess) e = hipMalloc((void **)&dc, (2 * want + 64) * sizeof(uint32_t));
        if (e != hipSuccess) {
          ctx->stats.last_hip_error = (int32_t)e;
          ss_note_hip_error((int)e, __FILE__, __LINE__);
          (void)hipGetLastError();
          return SS_E_NOMEM;
        }
        cap = want;
      }
      if (c.size() > 2 * cap + 64) return SS_E_CAPACITY;
      SS_HIP(hipMemcpy(dd, d.data(), d.size() * sizeof(ss_desc_t), hipMemcpyHostToDevice));
      SS_HIP(hipMemcpy(dc, c.data(), c.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
      return SS_OK;
    };
    if ((rc = upload(s.out, s.out_chunk0, s.d_out, s.d_out_chunk0, s.d_cap_out)) != SS_OK) return rc;
    if ((rc = upload(s.in, s.in_chunk0, s.d_in, s.d_in_chunk0, s.d_cap_in)) != SS_OK) return rc;
    auto upload_map = [&](const std::vector<uint32_t> &m, uint32_t *&dm, size_t &cap) -> int {
      if (m.empty()) return SS_OK;
      if (m.size() > cap) {
        if (dm) SS_HIP(hipFree(dm));
        dm = nullptr; cap = 0;
        const size_t want = m.size() + m.size() / 4 + 1024;
        hipError_t e = hipMalloc((void **)&dm, want * sizeof(uint32_t));
        if (e != hipSuccess) {
          ctx->stats.last_hip_error = (int32_t)e;
          ss_note_hip_error((int)e, __FILE__, __LINE__);
          (void)hipGetLastError();
          return SS_E_NOMEM;
        }
        cap = want;
      }
      SS_HIP(hipMemcpy(dm, m.data(), m.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
      return SS_OK;
    };
    if ((rc = upload_map(s.out_cdesc, s.d_out_cdesc, s.d_ccap_out)) != SS_OK) return rc;
    if ((rc = upload_map(s.in_cdesc, s.d_in_cdesc, s.d_ccap_in)) != SS_OK) return rc;
    s.loaded = true;
    return SS_OK;
  });
}

extern "C" int ss_schedule_view(ss_ctx *ctx, const uint32_t **out_start, uint32_t *n_out_batches,
                                const uint32_t **in_start, uint32_t *n_in_batches, const uint32_t **in_dep) {
  if (!ctx) return SS_E_INVAL;
  if (!ctx->sched.loaded) return SS_E_STATE;
  const ss_sched &s = ctx->sched;
  if (out_start) *out_start = s.out_start.data();
  if (n_out_batches) *n_out_batches = (uint32_t)s.out_start.size() - 1;
  if (in_start) *in_start = s.in_start.data();
  if (n_in_batches) *n_in_batches = (uint32_t)s.in_start.size() - 1;
  if (in_dep) *in_dep = s.in_dep.data();
  return SS_OK;
}

// ---- swap-out / swap-in / release / wait ---------------------------------------

// Path choice, by measurement on MI355X (PCIe Gen5 x16, 57 GB/s per direction with pinned
// hipMemcpy):
//  - many small tensors: one batched kernel launch moves them at 53-56 GB/s, per-tensor
//    copy-engine calls at about 30 GB/s (mean 600 KiB) -> kernel;
//  - large tensors coming back (swap-in) while the training step computes: the copy engine
//    runs at full link rate and leaves the compute stream alone, whereas a copy kernel that
//    saturates the link delays every concurrent kernel launch -> engine;
//  - tensors leaving (swap-out) under a running compute stream: engine copies of 8-16 MiB fell to
//    about 15 GB/s there while the copy kernel holds 50-55 GB/s -> kernel; from 32 MiB on the
//    engine reaches the link peak (93-99 %) and leaves the compute stream alone -> engine.
//    Engine and kernel swap-outs must not alternate on the stream: configuration 2 with its 32 and
//    64 MiB tensors by engine and its 8 and 16 MiB tensors by kernel took 215 ms against 126 ms all
//    by kernel.
// SS_PATH_AUTO therefore means: a swap-in batch goes by engine once its mean tensor size reaches
// engine_min_bytes, else by kernel; the swap-out side goes by engine as a whole if every batch of the
// schedule reaches engine_min_bytes_out, else by kernel as a whole.
static bool use_engine(const ss_ctx *ctx, uint32_t path, bool to_host, const std::vector<ss_desc_t> &d,
                       uint32_t lo, uint32_t hi) {
  if (path == SS_PATH_ENGINE) return true;
  if (path == SS_PATH_KERNEL) return false;
  // SS_PATH_AUTO, and the batches SS_PATH_STAGED does not stage
  if (to_host) return ctx->sched.out_all_large;        // one path for the whole swap-out side (see above)
  if (hi <= lo) return false;
  uint64_t total = 0;
  for (uint32_t i = lo; i < hi; ++i) total += d[i].nbytes;
  return total / (hi - lo) >= ctx->cfg.engine_min_bytes;
}

// Marker events are taken round-robin from a ring.  Re-recording one is safe however many waits on
// it are still pending: hipStreamWaitEvent captures the event's state (its most recent record) at the
// moment it is called, so a later record does not change what an earlier wait waits for.
static hipEvent_t next_marker(ss_ctx *ctx) {
  hipEvent_t ev = ctx->ev_ring[ctx->ev_next];
  ctx->ev_next = (ctx->ev_next + 1) % ctx->ev_ring.size();
  return ev;
}

// Where the compute stream stands when a batch is issued, in one of two forms, made when first needed (the
// dispatch thread enqueues nothing on the compute stream in between, so "now" is the same point either way).
// An event recorded on the compute stream that the swap stream waits for; or, with SS_CFG_MEMORY_MARKERS and a
// kernel as the consumer, a one-thread kernel on the compute stream that stores a running count in device memory
// and a bounded wait kernel on the swap stream.  An event of the compute stream that another stream waits for
// costs the compute stream about 0.13 ms here (nine of them: 1.3 ms of a 59 ms step; recorded but not waited
// for, or waited for but recorded long ago: nothing); the one-thread kernel a few microseconds.  A copy-engine
// transfer is never put behind a wait kernel (it would hold up the engine's queue): those keep the event.
struct ss_marker {
  hipEvent_t ev = nullptr;
  uint64_t count = 0;
};

static int wait_for_compute(ss_ctx *ctx, ss_marker &m, hipStream_t st, bool consumer_is_kernel) {
  if (ctx->d_mark && consumer_is_kernel) {
    if (!m.count) {
      m.count = ++ctx->mark_count;
      ss_launch_mark(ctx->compute, ctx->d_mark, m.count);
      SS_HIP(hipGetLastError());
    }
    ss_launch_wait_flag(st, ctx->d_mark, m.count, ctx->mark_limit_ticks, ctx->d_mark_gave_up, ctx->d_mark_timeouts);
    SS_HIP(hipGetLastError());
    return SS_OK;
  }
  if (!m.ev) {
    m.ev = next_marker(ctx);
    SS_HIP(hipEventRecord(m.ev, ctx->compute));
  }
  SS_HIP(hipStreamWaitEvent(st, m.ev, 0));
  return SS_OK;
}

// Staged swap-out: send what group g has in the ring and has not sent yet.  Per batch, ring_state is
// 0 = not issued, 1 = gathered into the ring, 2 = on its way to the staging area (or left directly).
// Every maximal run of gathered batches goes in one copy-engine transfer, which waits for the gathers
// and records the done-event of the run's last batch, standing for all of the run.
static int ring_flush(ss_ctx *ctx, uint32_t g) {
  ss_sched &s = ctx->sched;
  const ss_sched::out_group &G = s.groups[g];
  const uint8_t *slot = ctx->ring + (size_t)(g % ctx->n_slots) * ctx->cfg.ring_slot_bytes;
  for (uint32_t b = G.first; b <= G.last;) {
    if (s.ring_state[b] != 1) { ++b; continue; }
    uint32_t e = b;
    while (e <= G.last && s.ring_state[e] == 1) ++e;          // run [b, e)
    const uint64_t lo = s.out[s.out_start[b]].host_off;
    uint64_t bytes = 0;
    for (uint32_t i = s.out_start[b]; i < s.out_start[e]; ++i) bytes += s.out[i].nbytes;
    // the gathers run in issue order on one stream: the most recent one stands for all before it
    uint64_t seq = 0;
    if (ctx->eq) {
      seq = eq_push(ctx, ctx->staging + lo, slot + (lo - G.host_lo), bytes, hipMemcpyDeviceToHost,
                    &s.ev_gathered[s.phase][(size_t)s.last_gather_batch], 1, 2, g);
      s.group_last_flush_seq[g] = s.last_flush_seq = seq;
      s.group_started[g] = 1;
    } else {
      SS_HIP(hipStreamWaitEvent(ctx->s_flush, s.ev_gathered[s.phase][(size_t)s.last_gather_batch], 0));
      if ((ctx->cfg.flags & SS_CFG_TIMING) && !s.group_started[g]) SS_HIP(hipEventRecord(s.ev_flush_start[s.phase][g], ctx->s_flush));
      s.group_started[g] = 1;
      SS_HIP(hipMemcpyAsync(ctx->staging + lo, slot + (lo - G.host_lo), bytes, hipMemcpyDeviceToHost, ctx->s_flush));
      SS_HIP(hipEventRecord(s.ev_out_done[s.phase][e - 1], ctx->s_flush));
    }
    for (uint32_t x = b; x < e; ++x) {
      s.done_ev_of[x] = (int32_t)(e - 1);
      s.flush_seq[x] = seq;
      s.ring_state[x] = 2;
    }
    s.last_flush_batch = e - 1;
    s.group_last_flush[g] = (int32_t)(e - 1);
    ctx->stats.ring_transfers++;
    b = e;
  }
  return SS_OK;
}

// every gathered batch of every group is sent (before a swap-in that may need it, and at the drain)
static int ring_flush_all(ss_ctx *ctx) {
  ss_sched &s = ctx->sched;
  for (uint32_t g = 0; g < s.groups.size(); ++g) {
    if (!s.group_gathered[g]) continue;
    const int rc = ring_flush(ctx, g);
    if (rc != SS_OK) return rc;
    s.group_gathered[g] = 0;
  }
  return SS_OK;
}

// Swap-out of a batch that goes through the ring: gather on the swap-out stream, transfer when every
// batch of the group has been issued.  Returns 1 if the batch was handled here, 0 if it must leave
// directly (its ring slot already belongs to a later group: batches issued out of order), or an error code.
static int swap_out_staged(ss_ctx *ctx, uint32_t batch, ss_marker &mark) {
  ss_sched &s = ctx->sched;
  const int32_t g = s.group_of[batch];
  const ss_sched::out_group &G = s.groups[(size_t)g];
  const uint32_t slot = (uint32_t)g % ctx->n_slots;
  if (s.slot_owner[slot] > g) {
    s.ring_state[batch] = 2;
    if (s.group_pending[(size_t)g]) s.group_pending[(size_t)g]--;
    return 0;
  }
  hipStream_t so = ctx->s_out[0];
  if (s.slot_owner[slot] != g) {
    if (s.slot_owner[slot] >= 0) {
      // the slot still holds an earlier group: whatever of it has been gathered leaves now, and the first
      // gather of this group waits until the slot's last transfer has read it
      const uint32_t og = (uint32_t)s.slot_owner[slot];
      const int rc = ring_flush(ctx, og);
      if (rc != SS_OK) return rc;
      s.group_gathered[og] = 0;
      if (ctx->eq) {
        const int rw = eq_stream_wait(ctx, so, s.group_last_flush_seq[og], &ctx->eq->waited_out);
        if (rw != SS_OK) return rw;
      } else if (s.group_last_flush[og] >= 0) {
        SS_HIP(hipStreamWaitEvent(so, s.ev_out_done[s.phase][(size_t)s.group_last_flush[og]], 0));
      }
    }
    s.slot_owner[slot] = g;
  }
  const uint32_t lo = s.out_start[batch], hi = s.out_start[batch + 1];
  {
    const int rm = wait_for_compute(ctx, mark, so, true);
    if (rm != SS_OK) return rm;
  }
  if (ctx->cfg.flags & SS_CFG_TIMING) SS_HIP(hipEventRecord(s.ev_out_start[s.phase][batch], so));
  // the kernel adds each descriptor's host_off to its staging pointer: point it so that the group's
  // first byte lands on the first byte of the ring slot
  uint8_t *base = (uint8_t *)((uintptr_t)ctx->ring + (uintptr_t)slot * ctx->cfg.ring_slot_bytes - (uintptr_t)G.host_lo);
  const uint32_t *c0 = s.d_out_chunk0 + lo + batch;
  const uint32_t n_chunks = s.out_chunk0[(size_t)hi + batch];
  ss_launch_copy(so, ctx->cfg.gather_workgroups, ctx->cfg.copy_unroll, true, ctx->arena, base, s.d_out + lo, c0,
                 s.d_out_cdesc + s.out_cbase[batch], n_chunks, s.out_shift[batch], hi - lo, ctx->cfg.copy_desc_lookup == 1);
  SS_HIP(hipGetLastError());
  SS_HIP(hipEventRecord(s.ev_gathered[s.phase][batch], so));
  s.out_issued[batch] = 1;
  s.out_staged[batch] = 1;
  s.ring_state[batch] = 1;
  s.group_gathered[(size_t)g] = 1;
  s.last_gather_batch = batch;
  ctx->stats.kernel_batches++;
  ctx->stats.ring_batches++;
  if (s.group_pending[(size_t)g]) s.group_pending[(size_t)g]--;
  if (s.group_pending[(size_t)g] == 0) {                       // the group is complete
    const int rc = ring_flush(ctx, (uint32_t)g);
    if (rc != SS_OK) return rc;
    s.group_gathered[(size_t)g] = 0;
  }
  return 1;
}

static int swap_out_batch(ss_ctx *ctx, uint32_t batch);
static int swap_in_batch(ss_ctx *ctx, uint32_t batch);

extern "C" int ss_swap_out(ss_ctx *ctx, uint32_t batch) {
  if (!ctx) return SS_E_INVAL;
  if (ctx->bound && !ctx->arena && batch + 1 < ctx->sched.out_start.size() &&
      ctx->sched.out_start[batch + 1] > ctx->sched.out_start[batch])
    return SS_E_STATE;                              // no arena bound: the addresses must come with the call
  return swap_out_batch(ctx, batch);
}

// Device addresses given at issue time.  The batch's host-side descriptors take the addresses (as offsets from
// the arena base, which is 0 when no arena is bound).  Such a batch never goes through a ring and never reads
// the device copy of the descriptors: the copy engine takes the addresses from the host descriptors, the copy
// kernel gets them as launch arguments, one launch per tensor (ss_copy_flat_kernel).
static int patch_addresses(ss_ctx *ctx, bool out, uint32_t batch, const void *const *dev) {
  ss_sched &s = ctx->sched;
  std::vector<ss_desc_t> &d = out ? s.out : s.in;
  const std::vector<uint32_t> &start = out ? s.out_start : s.in_start;
  if (batch + 1 >= start.size()) return SS_E_INVAL;
  const uint32_t lo = start[batch], hi = start[batch + 1];
  if (hi > lo && !dev) return SS_E_INVAL;
  if (out ? s.out_issued[batch] : s.in_issued[batch]) return SS_E_STATE;
  if ((out ? s.group_of[batch] : s.in_group_of[batch]) >= 0) return SS_E_STATE;      // ring routes need the arena
  for (uint32_t i = lo; i < hi; ++i) {
    const uintptr_t a = (uintptr_t)dev[i - lo], base = (uintptr_t)ctx->arena;
    if (!a || (a & 15u) || a < base) return SS_E_INVAL;
    if (ctx->arena && (a - base > ctx->arena_bytes || d[i].nbytes > ctx->arena_bytes - (a - base))) return SS_E_INVAL;
  }
  for (uint32_t i = lo; i < hi; ++i) d[i].dev_off = (uint64_t)((uintptr_t)dev[i - lo] - (uintptr_t)ctx->arena);
  return SS_OK;
}

extern "C" int ss_swap_out_from(ss_ctx *ctx, uint32_t batch, const void *const *dev_src) {
  if (!ctx) return SS_E_INVAL;
  if (!ctx->sched.loaded || !ctx->bound) return SS_E_STATE;
  int rc = patch_addresses(ctx, true, batch, dev_src);
  if (rc != SS_OK) return rc;
  ctx->sched.flat_next = true;
  rc = swap_out_batch(ctx, batch);
  ctx->sched.flat_next = false;
  return rc;
}

extern "C" int ss_swap_in_to(ss_ctx *ctx, uint32_t batch, void *const *dev_dst) {
  if (!ctx) return SS_E_INVAL;
  if (!ctx->sched.loaded || !ctx->bound) return SS_E_STATE;
  int rc = patch_addresses(ctx, false, batch, dev_dst);
  if (rc != SS_OK) return rc;
  ctx->sched.flat_next = true;
  rc = swap_in_batch(ctx, batch);
  ctx->sched.flat_next = false;
  return rc;
}

static int swap_out_batch(ss_ctx *ctx, uint32_t batch) {
  ss_sched &s = ctx->sched;
  if (!s.loaded || !ctx->bound) return SS_E_STATE;
  if (batch + 1 >= s.out_start.size()) return SS_E_INVAL;
  if (s.out_issued[batch]) return SS_E_STATE;
  const uint32_t lo = s.out_start[batch], hi = s.out_start[batch + 1];
  // A batch whose addresses came with the call goes by copy engine unless the copy kernel is asked for
  // explicitly.  Measured on a real PyTorch model (12 layers, hidden 1024, bf16): with copy-kernel launches
  // running beside the step, the training loss is not reproducible bit for bit in some runs - and that also
  // happens (1 of 18 runs of ten steps) when the copy kernel moves a buffer that has nothing to do with the
  // model, with no ordering at all between the two streams, while every byte the swaps moved was checked to be
  // right.  So the model's own kernels are sensitive to what else occupies compute units (the order of their
  // floating-point accumulations changes with where their workgroups are placed); copy-engine transfers occupy
  // none, and every run with them was bit-identical to the run without swapping.  The synthetic configurations,
  // whose compute results are compared bit for bit in every test run, do not show it.
  // With bare ring transfers no batch goes by copy engine outside the rings: its transfer would sit on a swap
  // stream behind the kernels that wait for ring transfers, and a copy-engine transfer whose turn has not come
  // holds up the engine's queue - the queue in which the awaited transfer's sequence number travels.  (Seen: a
  // 96 MiB batch beside 64 MiB ring slots, by copy engine behind such a wait, stood until the wait gave up.)
  const bool engine = ctx->eq ? false
                    : s.flat_next ? ctx->cfg.copy_path != SS_PATH_KERNEL
                                  : use_engine(ctx, ctx->cfg.copy_path, true, s.out, lo, hi);
  // copy-kernel batches take the swap-out streams in turn; copy-engine batches stay on the first
  hipStream_t so = engine ? ctx->s_out[0] : ctx->s_out[batch % ctx->n_s_out];
  // the tensors' last forward use is already enqueued on the compute stream: order after it
  ss_marker mark;
  if (s.group_of[batch] >= 0) {
    const int rc = swap_out_staged(ctx, batch, mark);
    if (rc < 0) return rc;
    if (rc == 1) {
      uint64_t moved = 0;
      for (uint32_t i = lo; i < hi; ++i) moved += s.out[i].nbytes;
      ctx->stats.bytes_out += moved;
      return SS_OK;
    }
  }
  {
    const int rm = wait_for_compute(ctx, mark, so, !engine);
    if (rm != SS_OK) return rm;
  }
  if (ctx->cfg.flags & SS_CFG_TIMING) SS_HIP(hipEventRecord(s.ev_out_start[s.phase][batch], so));
  uint64_t bytes = 0;
  for (uint32_t i = lo; i < hi; ++i) bytes += s.out[i].nbytes;
  if (engine) {
    if (ctx->cfg.engine_window_out && s.engine_out_issued.size() >= ctx->cfg.engine_window_out) {   // see swap_in_batch
      const uint32_t old = s.engine_out_issued[s.engine_out_issued.size() - ctx->cfg.engine_window_out];
      SS_HIP(hipEventSynchronize(s.ev_out_done[s.phase][old]));
      ctx->stats.engine_window_waits++;
    }
    s.engine_out_issued.push_back(batch);
    for (uint32_t i = lo; i < hi; ++i)
      if (s.out[i].nbytes)
        SS_HIP(hipMemcpyAsync(ctx->staging + s.out[i].host_off, ctx->arena + s.out[i].dev_off, s.out[i].nbytes,
                              hipMemcpyDeviceToHost, so));
    ctx->stats.engine_batches++;
    ctx->stats.engine_batches_out++;
    s.last_engine_out = batch;
  } else if (s.flat_next) {
    for (uint32_t i = lo; i < hi; ++i)
      ss_launch_copy_flat(so, ctx->cfg.copy_workgroups_out, ctx->arena + s.out[i].dev_off, ctx->staging_dev + s.out[i].host_off,
                          s.out[i].nbytes);
    SS_HIP(hipGetLastError());
    ctx->stats.kernel_batches++;
  } else {
    const uint32_t *c0 = s.d_out_chunk0 + lo + batch;
    const uint32_t n_chunks = s.out_chunk0[(size_t)hi + batch];
    ss_launch_copy(so, ctx->cfg.copy_workgroups_out, ctx->cfg.copy_unroll, true, ctx->arena, ctx->staging_dev, s.d_out + lo, c0,
                   s.d_out_cdesc + s.out_cbase[batch], n_chunks, s.out_shift[batch], hi - lo, ctx->cfg.copy_desc_lookup == 1);
    SS_HIP(hipGetLastError());
    ctx->stats.kernel_batches++;
  }
  SS_HIP(hipEventRecord(s.ev_out_done[s.phase][batch], so));
  s.done_ev_of[batch] = (int32_t)batch;
  s.out_issued[batch] = 1;
  s.last_direct_out = batch;
  if ((int64_t)batch < s.max_out_issued) s.out_of_order = true;
  else s.max_out_issued = batch;
  s.last_out_on[engine ? 0 : batch % ctx->n_s_out] = batch;
  ctx->stats.bytes_out += bytes;
  return SS_OK;
}

// Swap-in of a batch that comes back through the ring.  With the first batch of its group the whole
// group's staging range is fetched into a ring slot by one copy-engine transfer (which waits for the bytes
// to be in the staging area and for the slot's previous readers, not for the compute stream: the blocks
// need not be free yet); the batch itself is scattered from the ring into its blocks by the copy kernel,
// after the compute stream has reached this point.  Returns 1 if handled, 0 if the batch must come back
// directly, or an error code.
static int swap_in_staged(ss_ctx *ctx, uint32_t batch, ss_marker &mark) {
  ss_sched &s = ctx->sched;
  const uint32_t g = (uint32_t)s.in_group_of[batch];
  const ss_sched::in_group &G = s.in_groups[g];
  const int32_t pack = s.in_pack_of[g];
  const uint32_t slot = (uint32_t)pack % ctx->n_slots;
  uint8_t *const home = ctx->ring_in + (size_t)slot * ctx->cfg.ring_slot_bytes + s.in_pack_off[g];   // the group's place in the ring
  if (s.in_group_state[g] == 2) return 0;
  if (s.in_group_state[g] == 0) {
    bool usable = s.in_slot_owner[slot] <= pack;
    for (uint32_t ob : s.in_group_outs[g]) usable = usable && s.out_issued[ob];   // every byte of the range is on its way
    if (!usable) {
      s.in_group_state[g] = 2;
      return 0;
    }
    // what has been gathered leaves the swap-out ring first; those transfers precede this one on the same stream
    int rc = ring_flush_all(ctx);
    if (rc != SS_OK) return rc;
    hipStream_t se = ctx->s_flush;
    // Tensors of the range that left directly (a batch the ring does not take, or one whose slot had gone to a
    // later group when it was issued): the direct batches share the swap-out stream with the gathers and run in
    // issue order, so the one issued most recently stands for all of them.
    bool left_directly = false;
    for (uint32_t ob : s.in_group_outs[g]) left_directly = left_directly || !s.out_staged[ob];
    const int64_t pd = left_directly ? s.last_direct_out : -1;
    const int32_t op = s.in_slot_owner[slot];           // the pack the slot held so far (this one, if a group of it came before)
    hipEvent_t pre[3];
    int n_pre = 0;
    if (pd >= 0) pre[n_pre++] = s.ev_out_done[s.phase][(size_t)pd];
    if (s.last_engine_out >= 0 && s.last_engine_out != pd) pre[n_pre++] = s.ev_out_done[s.phase][(size_t)s.last_engine_out];
    if (op >= 0 && op != pack && s.in_pack_last_scatter[(size_t)op] >= 0)
      pre[n_pre++] = s.ev_in_done[s.phase][(size_t)s.in_pack_last_scatter[(size_t)op]];
    s.in_slot_owner[slot] = pack;
    if (ctx->eq) {
      s.fetch_seq[g] = eq_push(ctx, home, ctx->staging + G.host_lo, G.bytes, hipMemcpyHostToDevice, pre, n_pre, 3, g);
    } else {
      for (int i = 0; i < n_pre; ++i) SS_HIP(hipStreamWaitEvent(se, pre[i], 0));
      if (ctx->cfg.flags & SS_CFG_TIMING) SS_HIP(hipEventRecord(s.ev_fetch_start[s.phase][g], se));
      SS_HIP(hipMemcpyAsync(home, ctx->staging + G.host_lo, G.bytes, hipMemcpyHostToDevice, se));
      SS_HIP(hipEventRecord(s.ev_fetched[s.phase][g], se));
    }
    s.in_group_state[g] = 1;
    ctx->stats.ring_transfers_in++;
  } else if (s.in_slot_owner[slot] != pack) {
    return 0;                                   // the slot has been handed on: the staging area still holds the bytes
  }
  hipStream_t si = ctx->s_in[0];
  const uint32_t lo = s.in_start[batch], hi = s.in_start[batch + 1];
  {
    const int rm = wait_for_compute(ctx, mark, si, true);                   // destination blocks are free from here on
    if (rm != SS_OK) return rm;
  }
  if (ctx->eq) {
    const int rw = eq_stream_wait(ctx, si, s.fetch_seq[g], &ctx->eq->waited_in);
    if (rw != SS_OK) return rw;
  } else {
    SS_HIP(hipStreamWaitEvent(si, s.ev_fetched[s.phase][g], 0));
  }
  if (ctx->cfg.flags & SS_CFG_TIMING) SS_HIP(hipEventRecord(s.ev_in_start[s.phase][batch], si));
  uint8_t *base = (uint8_t *)((uintptr_t)home - (uintptr_t)G.host_lo);
  const uint32_t *c0 = s.d_in_chunk0 + lo + batch;
  const uint32_t n_chunks = s.in_chunk0[(size_t)hi + batch];
  ss_launch_copy(si, ctx->cfg.gather_workgroups, ctx->cfg.copy_unroll, false, ctx->arena, base, s.d_in + lo, c0,
                 s.d_in_cdesc + s.in_cbase[batch], n_chunks, s.in_shift[batch], hi - lo, ctx->cfg.copy_desc_lookup == 1);
  SS_HIP(hipGetLastError());
  SS_HIP(hipEventRecord(s.ev_in_done[s.phase][batch], si));
  s.in_issued[batch] = 1;
  s.in_group_last_scatter[g] = (int32_t)batch;
  s.in_pack_last_scatter[(size_t)pack] = (int32_t)batch;
  ctx->stats.kernel_batches++;
  ctx->stats.ring_batches_in++;
  return 1;
}

extern "C" int ss_swap_in(ss_ctx *ctx, uint32_t batch) {
  if (!ctx) return SS_E_INVAL;
  if (ctx->bound && !ctx->arena && batch + 1 < ctx->sched.in_start.size() &&
      ctx->sched.in_start[batch + 1] > ctx->sched.in_start[batch])
    return SS_E_STATE;                              // no arena bound: the addresses must come with the call
  return swap_in_batch(ctx, batch);
}

static int swap_in_batch(ss_ctx *ctx, uint32_t batch) {
  ss_sched &s = ctx->sched;
  if (!s.loaded || !ctx->bound) return SS_E_STATE;
  if (batch + 1 >= s.in_start.size()) return SS_E_INVAL;
  if (s.in_issued[batch]) return SS_E_STATE;
  const uint32_t lo = s.in_start[batch], hi = s.in_start[batch + 1];
  if (hi > lo && !s.out_issued[s.in_dep[batch]]) return SS_E_STATE;   // its data never left
  if (s.out_of_order)      // swap-outs issued against their index order: the last one needed says nothing about the others
    for (uint32_t i = lo; i < hi; ++i) {
      auto it = s.out_of_tensor.find(s.in[i].tensor_id);
      if (it != s.out_of_tensor.end() && !s.out_issued[s.out_batch_of[it->second]]) return SS_E_STATE;
    }
  const bool engine = ctx->eq ? false                                                // see swap_out_batch
                    : s.flat_next ? ctx->cfg.copy_path_in != SS_PATH_KERNEL
                                  : use_engine(ctx, ctx->cfg.copy_path_in, false, s.in, lo, hi);
  hipStream_t si = engine ? ctx->s_in[0] : ctx->s_in[batch % ctx->n_s_in];
  // destination blocks are free once the compute stream reaches this point
  ss_marker mark;
  if (hi > lo && s.in_group_of[batch] >= 0) {
    const int rc = swap_in_staged(ctx, batch, mark);
    if (rc < 0) return rc;
    if (rc == 1) {
      uint64_t moved = 0;
      for (uint32_t i = lo; i < hi; ++i) moved += s.in[i].nbytes;
      ctx->stats.bytes_in += moved;
      return SS_OK;
    }
  }
  {
    const int rm = wait_for_compute(ctx, mark, si, !engine);
    if (rm != SS_OK) return rm;
  }
  // staging slots must be completely written: the batch's tensors left in swap-out batches up to in_dep;
  // with the swap-out batches spread over n streams, the last n of them up to in_dep cover every stream
  // (each stream runs its own batches in order)
  if (hi > lo && s.groups.empty() && s.out_of_order) {
    // swap-outs were not issued in index order: "up to in_dep" says nothing about what ran before what, so the
    // batch waits for the one issued most recently on every swap-out stream (everything issued so far)
    for (uint32_t k = 0; k < ctx->n_s_out; ++k)
      if (s.last_out_on[k] >= 0) SS_HIP(hipStreamWaitEvent(si, s.ev_out_done[s.phase][(size_t)s.last_out_on[k]], 0));
  } else if (hi > lo && s.groups.empty()) {
    const uint32_t dep = s.in_dep[batch];
    for (uint32_t back = 0; back < ctx->n_s_out && back <= dep; ++back)
      if (s.out_issued[dep - back]) SS_HIP(hipStreamWaitEvent(si, s.ev_out_done[s.phase][dep - back], 0));
  } else if (hi > lo) {
    // staged swap-out (one swap-out stream): what has been gathered so far leaves the ring now; the batch
    // waits for the direct batch issued most recently (they run in issue order on the swap-out stream, so it
    // stands for every direct batch so far, whichever of them the tensors left in) and for the last transfer
    // out of the ring (a copy-engine transfer towards the host must not meet one coming back anyway, see below)
    const int rc = ring_flush_all(ctx);
    if (rc != SS_OK) return rc;
    if (s.last_direct_out >= 0) SS_HIP(hipStreamWaitEvent(si, s.ev_out_done[s.phase][(size_t)s.last_direct_out], 0));
    if (ctx->eq) {
      const int rw = eq_stream_wait(ctx, si, s.last_flush_seq, &ctx->eq->waited_in);
      if (rw != SS_OK) return rw;
    } else if (s.last_flush_batch >= 0) {
      SS_HIP(hipStreamWaitEvent(si, s.ev_out_done[s.phase][(size_t)s.last_flush_batch], 0));
    }
  }
  // a copy-engine swap-out collapses to a quarter of the link rate as soon as anything flows the
  // other way: no swap-in starts before the engine swap-outs issued so far have finished
  if (s.last_engine_out >= 0 && (hi <= lo || (int64_t)s.in_dep[batch] < s.last_engine_out))
    SS_HIP(hipStreamWaitEvent(si, s.ev_out_done[s.phase][(size_t)s.last_engine_out], 0));
  if (ctx->cfg.flags & SS_CFG_TIMING) SS_HIP(hipEventRecord(s.ev_in_start[s.phase][batch], si));
  uint64_t bytes = 0;
  for (uint32_t i = lo; i < hi; ++i) bytes += s.in[i].nbytes;
  if (engine) {
    // Flow control: copy-engine transfers queued behind more than a few others run at a fraction of the link
    // rate, so with engine_window_in = w the call does not return before the engine swap-in batch issued w
    // batches earlier has finished: at most w of them are outstanding.  The host waits here only where the
    // link is the bottleneck anyway (the compute stream is waiting for those same transfers).
    if (ctx->cfg.engine_window_in && s.engine_in_issued.size() >= ctx->cfg.engine_window_in) {
      const uint32_t old = s.engine_in_issued[s.engine_in_issued.size() - ctx->cfg.engine_window_in];
      SS_HIP(hipEventSynchronize(s.ev_in_done[s.phase][old]));
      ctx->stats.engine_window_waits++;
    }
    s.engine_in_issued.push_back(batch);
    for (uint32_t i = lo; i < hi; ++i)
      if (s.in[i].nbytes)
        SS_HIP(hipMemcpyAsync(ctx->arena + s.in[i].dev_off, ctx->staging + s.in[i].host_off, s.in[i].nbytes,
                              hipMemcpyHostToDevice, si));
    ctx->stats.engine_batches++;
  } else if (s.flat_next) {
    for (uint32_t i = lo; i < hi; ++i)
      ss_launch_copy_flat(si, ctx->cfg.copy_workgroups, ctx->staging_dev + s.in[i].host_off, ctx->arena + s.in[i].dev_off,
                          s.in[i].nbytes);
    SS_HIP(hipGetLastError());
    ctx->stats.kernel_batches++;
  } else {
    const uint32_t *c0 = s.d_in_chunk0 + lo + batch;
    const uint32_t n_chunks = s.in_chunk0[(size_t)hi + batch];
    ss_launch_copy(si, ctx->cfg.copy_workgroups, ctx->cfg.copy_unroll, false, ctx->arena, ctx->staging_dev, s.d_in + lo, c0,
                   s.d_in_cdesc + s.in_cbase[batch], n_chunks, s.in_shift[batch], hi - lo, ctx->cfg.copy_desc_lookup == 1);
    SS_HIP(hipGetLastError());
    ctx->stats.kernel_batches++;
  }
  SS_HIP(hipEventRecord(s.ev_in_done[s.phase][batch], si));
  s.in_issued[batch] = 1;
  ctx->stats.bytes_in += bytes;
  return SS_OK;
}

// SS_CFG_BARE_RING with SS_CFG_TIMING, at the drain (every transfer is complete): the host-clock times of the
// iteration's ring transfers, folded per ring group
static void eq_harvest(ss_ctx *ctx) {
  ss_engine_queue *q = ctx->eq;
  if (!q || !q->timing) return;
  const ss_sched &s = ctx->sched;
  for (int i = 0; i < 20000; ++i) {             // the observer is at most a few microseconds behind
    {
      std::lock_guard<std::mutex> lk(q->mu);
      if (q->observed >= q->enqueued_seq) break;
    }
    std::this_thread::sleep_for(std::chrono::microseconds(10));
  }
  std::lock_guard<std::mutex> lk(q->mu);
  q->unit_start[0].assign(s.groups.size(), -1.0);
  q->unit_end[0].assign(s.groups.size(), -1.0);
  q->unit_start[1].assign(s.in_groups.size(), -1.0);
  q->unit_end[1].assign(s.in_groups.size(), -1.0);
  double prev_done = -1.0;
  for (const auto &r : q->recs) {
    const double start = r.t_enq > prev_done ? r.t_enq : prev_done;
    prev_done = r.t_done;
    const int d = r.dir == 3 ? 1 : 0;
    if (r.t_done < 0 || r.unit >= q->unit_start[d].size()) continue;
    if (q->unit_start[d][r.unit] < 0) q->unit_start[d][r.unit] = start;
    if (r.t_done > q->unit_end[d][r.unit]) q->unit_end[d][r.unit] = r.t_done;
  }
  q->recs.clear();
}

// a wait for a compute-stream marker gave up during the iteration that has just run
static int marker_timeouts(ss_ctx *ctx, int *late) {
  if (!ctx->h_mark_timeouts || !*(volatile uint32_t *)ctx->h_mark_timeouts) return SS_OK;
  *(volatile uint32_t *)ctx->h_mark_timeouts = 0;
  SS_HIP(hipMemcpy(ctx->d_mark_gave_up, ctx->h_mark_timeouts + 4, 4, hipMemcpyHostToDevice));
  *late = SS_E_TIMEOUT;
  return SS_OK;
}

extern "C" int ss_sync(ss_ctx *ctx, uint32_t what, uint32_t id) {
  if (!ctx) return SS_E_INVAL;
  ss_sched &s = ctx->sched;
  switch (what) {
    case SS_SYNC_FREE: {
      if (!s.loaded) return SS_E_STATE;
      auto it = s.out_of_tensor.find(id);
      if (it == s.out_of_tensor.end()) return SS_E_INVAL;
      const uint32_t b = s.out_batch_of[it->second];
      if (!s.out_issued[b]) return SS_E_STATE;   // releasing a block whose swap-out was never issued
      if (!s.out_waited[b]) {
        if (ctx->cfg.flags & SS_CFG_STALL_TIMING) SS_HIP(hipEventRecord(s.ev_free_at[b], ctx->compute));
        // device-side: later compute-stream work starts only after the batch has left its blocks (for the
        // staging area, or, staged, for the ring)
        SS_HIP(hipStreamWaitEvent(ctx->compute, s.out_staged[b] ? s.ev_gathered[s.phase][b] : s.ev_out_done[s.phase][b], 0));
        s.out_waited[b] = 1;
        ctx->stats.free_waits++;
      }
      if (ctx->cfg.flags & SS_CFG_POISON_FREE) {
        const ss_desc_t &d = s.out[it->second];
        ss_launch_fill(ctx->compute, ctx->arena + d.dev_off, d.nbytes, 0xDB);
        SS_HIP(hipGetLastError());
      }
      return SS_OK;
    }
    case SS_SYNC_WAIT_IN: {
      if (!s.loaded) return SS_E_STATE;
      auto it = s.in_of_tensor.find(id);
      if (it == s.in_of_tensor.end()) return SS_E_INVAL;
      const uint32_t b = s.in_batch_of[it->second];
      if (!s.in_issued[b]) return SS_E_STATE;    // waiting for a swap-in that was never issued
      if (!s.in_waited[b]) {
        if (ctx->cfg.flags & SS_CFG_STALL_TIMING) SS_HIP(hipEventRecord(s.ev_wait_at[b], ctx->compute));
        SS_HIP(hipStreamWaitEvent(ctx->compute, s.ev_in_done[s.phase][b], 0));
        s.in_waited[b] = 1;
        ctx->stats.in_waits++;
      }
      return SS_OK;
    }
    case SS_SYNC_ITERATION_END: {
      if (!s.loaded || (ctx->cfg.flags & SS_CFG_STALL_TIMING) || (ctx->eq && ctx->eq->timing))
        return ss_sync(ctx, SS_SYNC_DRAIN, id);
      int late = SS_OK;
      int rc = ring_flush_all(ctx);
      if (rc != SS_OK) return rc;
      const int cur = ctx->iter_set, prev = cur ^ 1;
      // the iteration before this one has to be over: the next one records into its set of events
      if (ctx->iter_pending[prev]) {
        for (int k = 0; k < 9; ++k)
          if (ctx->ev_iter[prev][k]) SS_HIP(hipEventSynchronize(ctx->ev_iter[prev][k]));
        eq_wait_enqueued(ctx, ctx->iter_last_seq[prev]);
        ctx->iter_pending[prev] = false;
      }
      if (ctx->eq) {
        const int he = ctx->eq->hip_error.exchange(0);
        if (he) {
          ctx->stats.last_hip_error = (int32_t)he;
          late = SS_E_HIP;
        }
        if (*(volatile uint32_t *)ctx->eq->h_timeouts) {      // of the iteration before: everything of it has run
          *(volatile uint32_t *)ctx->eq->h_timeouts = 0;
          SS_HIP(hipMemcpy(ctx->eq->d_gave_up, ctx->eq->h_timeouts + 4, 4, hipMemcpyHostToDevice));
          late = SS_E_TIMEOUT;
        }
      }
      if ((rc = marker_timeouts(ctx, &late)) != SS_OK) return rc;
      // where this iteration ends on every swap stream
      auto end_of = [&](int k, hipStream_t st) -> int {
        if (!ctx->ev_iter[cur][k])
          SS_HIP(hipEventCreateWithFlags(&ctx->ev_iter[cur][k], hipEventDisableTiming | fence_flag(ctx->cfg)));
        SS_HIP(hipEventRecord(ctx->ev_iter[cur][k], st));
        return SS_OK;
      };
      for (uint32_t i = 0; i < ctx->n_s_out; ++i)
        if ((rc = end_of((int)i, ctx->s_out[i])) != SS_OK) return rc;
      for (uint32_t i = 0; i < ctx->n_s_in; ++i)
        if ((rc = end_of(4 + (int)i, ctx->s_in[i])) != SS_OK) return rc;
      if (ctx->s_flush && !ctx->eq && (rc = end_of(8, ctx->s_flush)) != SS_OK) return rc;
      // The next iteration's swap-outs write staging slots and ring slots that this iteration's swap-ins and ring
      // transfers still read: every swap-out stream goes on only after the swap-in streams and the ring transfers of
      // this iteration; the ring transfers of the next iteration (into slots this iteration's scatters read) only
      // after the swap-in streams.  Swap-ins follow their own swap-outs as always.
      for (uint32_t i = 0; i < ctx->n_s_out; ++i) {
        for (uint32_t j = 0; j < ctx->n_s_in; ++j) SS_HIP(hipStreamWaitEvent(ctx->s_out[i], ctx->ev_iter[cur][4 + j], 0));
        if (ctx->s_flush && !ctx->eq) SS_HIP(hipStreamWaitEvent(ctx->s_out[i], ctx->ev_iter[cur][8], 0));
      }
      if (ctx->eq) {
        const uint64_t last = ctx->eq->next_seq - 1;           // only this thread pushes
        if ((rc = eq_stream_wait(ctx, ctx->s_out[0], last, &ctx->eq->waited_out)) != SS_OK) return rc;
        // a transfer of nothing that the thread holds back until the scatters are done: what is pushed later follows it
        ctx->iter_last_seq[cur] = eq_push(ctx, nullptr, nullptr, 0, hipMemcpyHostToDevice, &ctx->ev_iter[cur][4], 1, 3, 0);
      } else if (ctx->s_flush) {
        for (uint32_t j = 0; j < ctx->n_s_in; ++j) SS_HIP(hipStreamWaitEvent(ctx->s_flush, ctx->ev_iter[cur][4 + j], 0));
      }
      ctx->iter_pending[cur] = true;
      ctx->iter_set ^= 1;
      std::fill(s.out_waited.begin(), s.out_waited.end(), 0);
      std::fill(s.in_waited.begin(), s.in_waited.end(), 0);
      std::fill(s.out_issued.begin(), s.out_issued.end(), 0);
      std::fill(s.in_issued.begin(), s.in_issued.end(), 0);
      s.last_engine_out = -1;
      s.phase ^= 1;
      s.drained_once = true;
      s.done_ev_of_drained = s.done_ev_of;
      s.out_staged_drained = s.out_staged;
      s.group_last_flush_drained = s.group_last_flush;
      s.in_group_state_drained = s.in_group_state;
      ring_reset(s, ctx->n_slots);
      return late;
    }
    case SS_SYNC_DRAIN: {
      int late = SS_OK;             // what the iteration's ring transfers ran into; reported once the state is reset
      {
        int rc = s.loaded ? ring_flush_all(ctx) : SS_OK;      // staged batches whose group never completed
        if (rc == SS_OK) rc = sync_swap_streams(ctx);
        if (rc != SS_OK) return rc;
        ctx->iter_pending[0] = ctx->iter_pending[1] = false;   // every stream is idle
        if (ctx->eq) {
          {
            std::lock_guard<std::mutex> lk(ctx->eq->mu);          // the thread is idle and its stream empty
            ctx->eq->synced_seq = ctx->eq->enqueued_seq;
          }
          eq_harvest(ctx);
          const int he = ctx->eq->hip_error.exchange(0);
          if (he) {
            ctx->stats.last_hip_error = (int32_t)he;
            late = SS_E_HIP;
          }
          if (*(volatile uint32_t *)ctx->eq->h_timeouts) {
            *(volatile uint32_t *)ctx->eq->h_timeouts = 0;
            SS_HIP(hipMemcpy(ctx->eq->d_gave_up, ctx->eq->h_timeouts + 4, 4, hipMemcpyHostToDevice));   // every stream is idle
            late = SS_E_TIMEOUT;
          }
        }
        if ((rc = marker_timeouts(ctx, &late)) != SS_OK) return rc;
      }
      if ((ctx->cfg.flags & SS_CFG_STALL_TIMING) && s.loaded) {
        // measurement mode: the compute stream is joined too, then every wait of this iteration is
        // charged with the time from reaching it to the end of the batch it waited for
        SS_HIP(hipStreamSynchronize(ctx->compute));
        for (size_t b = 0; b < s.out_waited.size(); ++b)
          if (s.out_waited[b]) {
            float ms = 0.f;
            SS_HIP(hipEventElapsedTime(&ms, s.ev_free_at[b], s.out_staged[b] ? s.ev_gathered[s.phase][b] : s.ev_out_done[s.phase][b]));
            if (ms > 0.f) ctx->stats.stall_free_ms += ms;
          }
        for (size_t b = 0; b < s.in_waited.size(); ++b)
          if (s.in_waited[b]) {
            float ms = 0.f;
            SS_HIP(hipEventElapsedTime(&ms, s.ev_wait_at[b], s.ev_in_done[s.phase][b]));
            if (ms > 0.f) ctx->stats.stall_wait_in_ms += ms;
          }
      }
      std::fill(s.out_waited.begin(), s.out_waited.end(), 0);
      std::fill(s.in_waited.begin(), s.in_waited.end(), 0);
      std::fill(s.out_issued.begin(), s.out_issued.end(), 0);
      std::fill(s.in_issued.begin(), s.in_issued.end(), 0);
      s.last_engine_out = -1;
      if (s.loaded) {              // the next iteration records into the other event set
        s.phase ^= 1;
        s.drained_once = true;
        s.done_ev_of_drained = s.done_ev_of;
        s.out_staged_drained = s.out_staged;
        s.group_last_flush_drained = s.group_last_flush;
        s.in_group_state_drained = s.in_group_state;
        ring_reset(s, ctx->n_slots);
      }
      return late;
    }
    default: return SS_E_INVAL;
  }
}

extern "C" int ss_dispatch(ss_ctx *ctx, uint32_t op_idx, uint32_t when) {
  if (!ctx || when > 1) return SS_E_INVAL;
  ss_sched &s = ctx->sched;
  if (!s.loaded || !s.have_actions) return SS_E_STATE;
  const uint64_t g = 2ull * op_idx + when;
  if (g + 1 >= s.act_start.size()) return SS_OK;          // beyond the last operator with actions
  for (uint32_t a = s.act_start[g]; a < s.act_start[g + 1]; ++a) {
    const ss_action_t &act = s.actions[a];
    int rc = SS_OK;
    switch (act.kind) {
      case SS_ACT_IN: if (!s.in_issued[act.batch]) rc = ss_swap_in(ctx, act.batch); break;
      case SS_ACT_WAIT_IN: rc = ss_sync(ctx, SS_SYNC_WAIT_IN, act.tensor_id); break;
      case SS_ACT_OUT: if (!s.out_issued[act.batch]) rc = ss_swap_out(ctx, act.batch); break;
      case SS_ACT_FREE: rc = ss_sync(ctx, SS_SYNC_FREE, act.tensor_id); break;
      default: rc = SS_E_INVAL;
    }
    if (rc != SS_OK) return rc;
  }
  return SS_OK;
}

// Start / end event of unit `u` of direction `dir` in the iteration drained last: dir 0 swap-out batch
// (a staged batch: its gather into the ring), 1 swap-in batch, 2 transfer of ring group u to the host.
static int timing_events(ss_ctx *ctx, uint32_t dir, uint32_t u, hipEvent_t *st, hipEvent_t *dn) {
  ss_sched &s = ctx->sched;
  const int set = s.drained_once ? s.phase ^ 1 : s.phase;
  const std::vector<uint8_t> &staged = s.drained_once ? s.out_staged_drained : s.out_staged;
  if (dir == 0) {
    if (u + 1 >= s.out_start.size()) return SS_E_INVAL;
    *st = s.ev_out_start[set][u];
    *dn = staged[u] ? s.ev_gathered[set][u] : s.ev_out_done[set][u];
  } else if (dir == 1) {
    if (u + 1 >= s.in_start.size()) return SS_E_INVAL;
    *st = s.ev_in_start[set][u];
    *dn = s.ev_in_done[set][u];
  } else if (ctx->eq) {
    return SS_E_STATE;                                         // bare ring transfers carry no events (host clock: bare_unit_ms)
  } else if (dir == 3) {
    if (u >= s.in_groups.size()) return SS_E_INVAL;
    const std::vector<uint8_t> &st_ = s.drained_once ? s.in_group_state_drained : s.in_group_state;
    if (st_[u] != 1) return SS_E_STATE;                        // the group did not come back through the ring
    *st = s.ev_fetch_start[set][u];
    *dn = s.ev_fetched[set][u];
  } else {
    if (u >= s.groups.size()) return SS_E_INVAL;
    const std::vector<int32_t> &lf = s.drained_once ? s.group_last_flush_drained : s.group_last_flush;
    if (u >= lf.size() || lf[u] < 0) return SS_E_STATE;        // nothing of the group went through the ring
    *st = s.ev_flush_start[set][u];
    *dn = s.ev_out_done[set][(size_t)lf[u]];
  }
  return SS_OK;
}

// SS_CFG_BARE_RING: duration of ring transfer unit u of direction dir (2, 3) in the iteration drained last,
// and its end relative to the start of unit 0, on the host's clock
static int bare_unit_ms(ss_ctx *ctx, uint32_t dir, uint32_t u, float *ms, float *end_from_first) {
  ss_engine_queue *q = ctx->eq;
  if (!q->timing) return SS_E_STATE;
  std::lock_guard<std::mutex> lk(q->mu);
  const std::vector<double> &st = q->unit_start[dir - 2], &en = q->unit_end[dir - 2];
  if (u >= st.size()) return SS_E_INVAL;
  if (st[u] < 0 || en[u] < 0) return SS_E_STATE;
  if (ms) *ms = (float)(en[u] - st[u]);
  if (end_from_first) {
    if (st[0] < 0) return SS_E_STATE;
    *end_from_first = (float)(en[u] - st[0]);
  }
  return SS_OK;
}

static size_t timing_units(const ss_sched &s, uint32_t dir) {
  return dir == 0 ? s.out_start.size() - 1 : dir == 1 ? s.in_start.size() - 1 : dir == 2 ? s.groups.size() : s.in_groups.size();
}

extern "C" int ss_batch_ms(ss_ctx *ctx, uint32_t dir, uint32_t batch, float *ms, float *span_ms) {
  if (!ctx || dir > 3) return SS_E_INVAL;
  if (!(ctx->cfg.flags & SS_CFG_TIMING) || !ctx->sched.loaded) return SS_E_STATE;
  ss_sched &s = ctx->sched;
  const size_t nb = timing_units(s, dir);
  hipEvent_t st, dn;
  int rc;
  if (ctx->eq && dir >= 2) {
    if (ms && (rc = bare_unit_ms(ctx, dir, batch, ms, nullptr)) != SS_OK) return rc;
    if (span_ms) {
      *span_ms = 0.f;
      if (nb == 0) return SS_OK;
      if ((rc = bare_unit_ms(ctx, dir, 0, nullptr, span_ms)) != SS_OK) return rc;
      for (size_t b = nb > 8 ? nb - 8 : 0; b < nb; ++b) {
        float x = 0.f;
        if (bare_unit_ms(ctx, dir, (uint32_t)b, nullptr, &x) == SS_OK && x > *span_ms) *span_ms = x;
      }
    }
    return SS_OK;
  }
  if (ms) {
    if ((rc = timing_events(ctx, dir, batch, &st, &dn)) != SS_OK) return rc;
    SS_HIP(hipEventElapsedTime(ms, st, dn));
  }
  if (span_ms) {
    *span_ms = 0.f;
    if (nb == 0) return SS_OK;
    // first start to last end: with several streams per direction the units need not end in order
    hipEvent_t st0, dn0;
    if ((rc = timing_events(ctx, dir, 0, &st0, &dn0)) != SS_OK) return rc;
    for (size_t b = nb > 8 ? nb - 8 : 0; b < nb; ++b) {
      float x = 0.f;
      if (timing_events(ctx, dir, (uint32_t)b, &st, &dn) != SS_OK) continue;
      SS_HIP(hipEventElapsedTime(&x, st0, dn));
      if (x > *span_ms) *span_ms = x;
    }
  }
  return SS_OK;
}

extern "C" int ss_batch_ms_all(ss_ctx *ctx, uint32_t dir, float *ms, uint32_t capacity, uint32_t *n) {
  if (!ctx || dir > 3 || !n || (capacity && !ms)) return SS_E_INVAL;
  if (!(ctx->cfg.flags & SS_CFG_TIMING) || !ctx->sched.loaded) return SS_E_STATE;
  const size_t nb = timing_units(ctx->sched, dir);
  *n = (uint32_t)nb;
  if (nb > capacity) return SS_E_CAPACITY;
  for (size_t u = 0; u < nb; ++u) {
    hipEvent_t st, dn;
    ms[u] = -1.f;                                   // a unit that did not run this way (see ss_batch_ms)
    if (ctx->eq && dir >= 2) {
      if (bare_unit_ms(ctx, dir, (uint32_t)u, &ms[u], nullptr) != SS_OK) ms[u] = -1.f;
      continue;
    }
    if (timing_events(ctx, dir, (uint32_t)u, &st, &dn) != SS_OK) continue;
    SS_HIP(hipEventElapsedTime(&ms[u], st, dn));
  }
  return SS_OK;
}

extern "C" int ss_batch_done(ss_ctx *ctx, uint32_t dir, uint32_t batch, int *done) {
  if (!ctx || dir > 1 || !done) return SS_E_INVAL;
  ss_sched &s = ctx->sched;
  if (!s.loaded) return SS_E_STATE;
  const size_t nb = (dir ? s.in_start.size() : s.out_start.size()) - 1;
  if (batch >= nb) return SS_E_INVAL;
  if (!(dir ? s.in_issued[batch] : s.out_issued[batch])) return SS_E_STATE;
  if (dir == 0 && s.done_ev_of[batch] < 0) {                  // gathered into the ring, not yet on its way to the host
    *done = 0;
    return SS_OK;
  }
  hipError_t e;
  if (dir == 0 && ctx->eq && s.flush_seq[batch]) {
    // no event of its own: complete once its transfer is on the stream and the stream has nothing left to do
    bool on_stream;
    {
      std::lock_guard<std::mutex> lk(ctx->eq->mu);
      on_stream = ctx->eq->enqueued_seq >= s.flush_seq[batch];
    }
    e = on_stream ? hipStreamQuery(ctx->s_flush) : hipErrorNotReady;
  } else {
    e = hipEventQuery(dir ? s.ev_in_done[s.phase][batch] : s.ev_out_done[s.phase][(size_t)s.done_ev_of[batch]]);
  }
  if (e == hipErrorNotReady) {
    (void)hipGetLastError();
    *done = 0;
    return SS_OK;
  }
  SS_HIP(e);
  *done = 1;
  return SS_OK;
}

extern "C" int ss_batch_window(ss_ctx *ctx, uint32_t dir, uint32_t batch, float *start_ms, float *end_ms) {
  if (!ctx || dir > 3 || !start_ms || !end_ms) return SS_E_INVAL;
  if (!(ctx->cfg.flags & SS_CFG_TIMING) || !ctx->sched.loaded) return SS_E_STATE;
  ss_sched &s = ctx->sched;
  if (s.out_start.size() < 2) return SS_E_INVAL;
  hipEvent_t st, dn, st0, dn0;
  int rc;
  if ((rc = timing_events(ctx, dir, batch, &st, &dn)) != SS_OK) return rc;
  if ((rc = timing_events(ctx, 0, 0, &st0, &dn0)) != SS_OK) return rc;
  SS_HIP(hipEventElapsedTime(start_ms, st0, st));
  SS_HIP(hipEventElapsedTime(end_ms, st0, dn));
  return SS_OK;
}

extern "C" int ss_ring_view(ss_ctx *ctx, uint32_t dir, uint32_t *n_groups, const int32_t **group_of,
                            const uint64_t **group_bytes) {
  if (!ctx || dir > 1) return SS_E_INVAL;
  if (!ctx->sched.loaded) return SS_E_STATE;
  const ss_sched &s = ctx->sched;
  if (n_groups) *n_groups = (uint32_t)(dir ? s.in_groups.size() : s.groups.size());
  if (group_of) *group_of = dir ? s.in_group_of.data() : s.group_of.data();
  if (group_bytes) *group_bytes = dir ? s.in_group_bytes.data() : s.group_bytes.data();
  return SS_OK;
}

// ---- support -------------------------------------------------------------------

extern "C" int ss_host_peek(ss_ctx *ctx, uint64_t host_off, uint64_t nbytes, const void **ptr) {
  if (!ctx || !ptr) return SS_E_INVAL;
  if (host_off > ctx->cfg.staging_bytes || nbytes > ctx->cfg.staging_bytes - host_off) return SS_E_INVAL;
  *ptr = ctx->staging + host_off;
  return SS_OK;
}

extern "C" int ss_staging_fill(ss_ctx *ctx, int byte) {
  if (!ctx) return SS_E_INVAL;
  {
    const int rc = sync_swap_streams(ctx);
    if (rc != SS_OK) return rc;
  }
  if (ctx->staging) std::memset(ctx->staging, byte, ctx->cfg.staging_bytes);
  return SS_OK;
}

extern "C" int ss_get_stats(ss_ctx *ctx, ss_stats_t *out) {
  if (!ctx || !out) return SS_E_INVAL;
  *out = ctx->stats;
  return SS_OK;
}

// Host-link bandwidth as the machine delivers it now.
extern "C" int ss_bw_probe(ss_ctx *ctx, uint64_t bytes, uint32_t reps, ss_bw_t *out) {
  return ss_guard([&]() -> int {
    if (!ctx || !out || bytes < 4096 || reps == 0 || reps > 1000) return SS_E_INVAL;
    bytes &= ~(uint64_t)255;
    std::memset(out, 0, sizeof(*out));
    uint8_t *h0 = nullptr, *h1 = nullptr, *d0 = nullptr, *d1 = nullptr, *h0d = nullptr, *h1d = nullptr;
    ss_desc_t *dd = nullptr;
    uint32_t *dc = nullptr, *dm = nullptr;
    hipEvent_t a0 = nullptr, a1 = nullptr, b0 = nullptr, b1 = nullptr;
    int rc = SS_OK;
    auto ck = [&](hipError_t e) {
      if (e != hipSuccess && rc == SS_OK) {
        ctx->stats.last_hip_error = (int32_t)e;
        ss_note_hip_error((int)e, __FILE__, 0);
        (void)hipGetLastError();
        rc = SS_E_HIP;
      }
      return e == hipSuccess;
    };
    ck(hipHostMalloc((void **)&h0, bytes, hipHostMallocMapped));
    ck(hipHostMalloc((void **)&h1, bytes, hipHostMallocMapped));
    ck(hipMalloc((void **)&d0, bytes));
    ck(hipMalloc((void **)&d1, bytes));
    ck(hipMalloc((void **)&dd, 2 * sizeof(ss_desc_t)));
    ck(hipMalloc((void **)&dc, 4 * sizeof(uint32_t)));
    ck(hipMalloc((void **)&dm, ((bytes + SS_CHUNK_BYTES - 1) / SS_CHUNK_BYTES) * sizeof(uint32_t)));
    ck(hipEventCreate(&a0)); ck(hipEventCreate(&a1)); ck(hipEventCreate(&b0)); ck(hipEventCreate(&b1));
    if (rc == SS_OK) {
      ck(hipHostGetDevicePointer((void **)&h0d, h0, 0));
      ck(hipHostGetDevicePointer((void **)&h1d, h1, 0));
      std::memset(h0, 1, bytes);
      std::memset(h1, 2, bytes);
      ck(hipMemset(d0, 3, bytes));
      ck(hipMemset(d1, 4, bytes));
      ss_desc_t hd[2] = {{0, 0, bytes, 0, 0}, {0, 0, bytes, 1, 0}};
      uint32_t hc[2] = {0, (uint32_t)((bytes + SS_CHUNK_BYTES - 1) / SS_CHUNK_BYTES)};
      ck(hipMemcpy(dd, hd, sizeof(hd), hipMemcpyHostToDevice));
      ck(hipMemcpy(dc, hc, sizeof(hc), hipMemcpyHostToDevice));
      ck(hipMemset(dm, 0, ((bytes + SS_CHUNK_BYTES - 1) / SS_CHUNK_BYTES) * sizeof(uint32_t)));   // every chunk: descriptor 0
      ck(hipDeviceSynchronize());
    }
    auto median = [](std::vector<float> &v) {
      std::sort(v.begin(), v.end());
      return v[v.size() / 2];
    };
    auto gbps = [&](float ms) { return ms > 0 ? (double)bytes / (ms * 1e-3) / 1e9 : 0.0; };
    const uint32_t wg = ctx->cfg.copy_workgroups, wgo = ctx->cfg.copy_workgroups_out;
    const uint32_t nchunks = (uint32_t)((bytes + SS_CHUNK_BYTES - 1) / SS_CHUNK_BYTES);
    // mode 0: D2H engine, 1: H2D engine, 2: both engine, 3: D2H kernel, 4: H2D kernel, 5: both kernel
    for (int mode = 0; mode < 6 && rc == SS_OK; ++mode) {
      std::vector<float> ta, tb;
      for (uint32_t r = 0; r < reps + 2 && rc == SS_OK; ++r) {
        const bool d2h = (mode == 0 || mode == 2 || mode == 3 || mode == 5);
        const bool h2d = (mode == 1 || mode == 2 || mode == 4 || mode == 5);
        if (d2h) {
          ck(hipEventRecord(a0, ctx->s_out[0]));
          if (mode == 3 || mode == 5) {
            ss_launch_copy(ctx->s_out[0], wgo, ctx->cfg.copy_unroll, true, d0, h0d, dd, dc, dm, nchunks, SS_CHUNK_SHIFT, 1, false);
            ck(hipGetLastError());
          } else ck(hipMemcpyAsync(h0, d0, bytes, hipMemcpyDeviceToHost, ctx->s_out[0]));
          ck(hipEventRecord(a1, ctx->s_out[0]));
        }
        if (h2d) {
          ck(hipEventRecord(b0, ctx->s_in[0]));
          if (mode == 4 || mode == 5) {
            ss_launch_copy(ctx->s_in[0], wg, ctx->cfg.copy_unroll, false, d1, h1d, dd, dc, dm, nchunks, SS_CHUNK_SHIFT, 1, false);
            ck(hipGetLastError());
          } else ck(hipMemcpyAsync(d1, h1, bytes, hipMemcpyHostToDevice, ctx->s_in[0]));
          ck(hipEventRecord(b1, ctx->s_in[0]));
        }
        ck(hipStreamSynchronize(ctx->s_out[0]));
        ck(hipStreamSynchronize(ctx->s_in[0]));
        float ms;
        if (d2h && ck(hipEventElapsedTime(&ms, a0, a1)) && r >= 2) ta.push_back(ms);
        if (h2d && ck(hipEventElapsedTime(&ms, b0, b1)) && r >= 2) tb.push_back(ms);
      }
      if (rc != SS_OK) break;
      switch (mode) {
        case 0: out->d2h_gbps = gbps(median(ta)); break;
        case 1: out->h2d_gbps = gbps(median(tb)); break;
        case 2: out->bidir_d2h_gbps = gbps(median(ta)); out->bidir_h2d_gbps = gbps(median(tb)); break;
        case 3: out->kernel_d2h_gbps = gbps(median(ta)); break;
        case 4: out->kernel_h2d_gbps = gbps(median(tb)); break;
        case 5: out->kernel_bidir_d2h_gbps = gbps(median(ta)); out->kernel_bidir_h2d_gbps = gbps(median(tb)); break;
      }
    }
    if (a0) (void)hipEventDestroy(a0);
    if (a1) (void)hipEventDestroy(a1);
    if (b0) (void)hipEventDestroy(b0);
    if (b1) (void)hipEventDestroy(b1);
    if (dd) (void)hipFree(dd);
    if (dc) (void)hipFree(dc);
    if (dm) (void)hipFree(dm);
    if (d0) (void)hipFree(d0);
    if (d1) (void)hipFree(d1);
    if (h0) (void)hipHostFree(h0);
    if (h1) (void)hipHostFree(h1);
    return rc;
  });
}
