// Memory-timeline scan on the GPU (Sec. 3 last paragraph and Sec. 4.2 of the SmartSwap
// paper): from the alloc/free trace of an iteration, plus the releases and allocations a
// swap policy induces, compute the memory in use at every operator, its peak, and the
// memory reduction entries (excess over the budget per operator).
//
// One workgroup of 1024 lanes handles one scan: per-operator class sums are gathered
// with 64-bit integer atomics (order-independent, hence deterministic), a chunked
// workgroup prefix scan over the operators gives the amount held on entry to each
// operator, and, if the per-event timeline is wanted, a second chunked scan over each
// event list places every event at its canonical position.  At the sizes of a training
// iteration (thousands of operators, up to 10^5 events) the work is latency-bound;
// keeping one scan inside one workgroup makes a batch of scans (one per candidate
// policy) a single launch.
#include <algorithm>
#include <cstring>

#include "ss_internal.h"

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;

struct ScanArgs {
  const ss_event_t *ev;    uint64_t n_ev;
  const ss_event_t *pev;   uint64_t n_pe;
  uint32_t n_ops;          int want_timeline;
  int64_t base, budget;
  // scratch
  int64_t *csum;    // [4][n_ops] sum of deltas per (class, operator)
  uint32_t *ccnt;   // [4][n_ops] number of events per (class, operator)
  int64_t *before;  // [n_ops] total held on entry to the operator, without base
  uint32_t *evstart;// [n_ops] canonical position of the operator's first event
  int64_t *segsum;  // [4][n_ops] running class sum of the own list at the operator's first event
  uint32_t *segcnt; // [4][n_ops]
  int64_t *sumx;    // [n_ev + n_pe] exclusive running sum of the event's own class in its list
  uint32_t *cntx;   // [n_ev + n_pe]
  // outputs
  int64_t *per_op, *mre, *timeline;
  ss_scan_result_t *res;
  uint32_t *flags;  // bit 0: event names an operator >= n_ops; bit 1: a list is not in operator order
  int res_flags;    // also report the flags in res->reserved (for callers that read nothing but res)
};

__device__ inline int64_t shfl_up_i64(int64_t v, int d) {
  int lo = __shfl_up((int)(uint32_t)(uint64_t)v, d, 64);
  int hi = __shfl_up((int)(uint32_t)((uint64_t)v >> 32), d, 64);
  return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

// Inclusive prefix sum over the workgroup (lane order = threadIdx.x); returns the
// inclusive value and the workgroup total.  `wsum` holds one entry per wavefront.
__device__ inline int64_t block_scan_i64(int64_t v, int64_t *wsum, int64_t &total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    int64_t o = shfl_up_i64(v, d);
    if (lane >= d) v += o;
  }
  __syncthreads();               // wsum may still be read from the previous call
  if (lane == 63) wsum[w] = v;
  __syncthreads();
  int64_t add = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kWaves; ++i) {
    int64_t x = wsum[i];
    if (i < w) add += x;
    tot += x;
  }
  total = tot;
  return v + add;
}

__device__ inline void add_i64(int64_t *p, int64_t v) {
  atomicAdd(reinterpret_cast<unsigned long long *>(p), (unsigned long long)v);
}

// class of an event: 0 policy alloc, 1 trace alloc, 2 trace release, 3 policy release
__device__ inline int event_class(bool policy, int64_t delta) {
  return policy ? (delta >= 0 ? 0 : 3) : (delta >= 0 ? 1 : 2);
}

// phase 1: gather class sums and counts per operator (integer atomics: any order, same result).
// Neighbouring events mostly belong to the same operator, and 64 lanes adding to one address are
// served one after the other: so each wavefront first folds every run of equal operators among its
// 64 consecutive events (two wavefront prefix sums, two ballots) and only the first lane of a run
// adds the run's totals.  Workgroup `wg` of `n_wg` takes every n_wg-th stretch of events; the
// accumulators must have been cleared before any workgroup starts.  Returns this lane's share of the
// flags (bit 0: operator out of range, bit 1: list not in operator order).
__device__ __forceinline__ uint32_t gather_events(const ScanArgs &a, uint32_t wg, uint32_t n_wg) {
  const uint32_t tid = threadIdx.x;
  const uint32_t n = a.n_ops;
  uint32_t bad = 0;
  const int lane = tid & 63;
  const uint64_t below = lane ? (~0ull >> (64 - lane)) : 0ull;           // bits of the lanes before this one
  for (int list = 0; list < 2; ++list) {
    const ss_event_t *L = list ? a.pev : a.ev;
    const uint64_t cnt = list ? a.n_pe : a.n_ev;
    const int cpos = list ? 0 : 1, cneg = list ? 3 : 2;
    constexpr int kAhead = 4;            // events in flight per lane: the loop is bound by load latency
    for (uint64_t g0 = (uint64_t)wg * kAhead * kThreads; g0 < cnt; g0 += (uint64_t)n_wg * kAhead * kThreads) {
      ss_event_t xs[kAhead];
      uint32_t before0[kAhead];          // lane 0 only: operator of the event before the wavefront's first
#pragma unroll
      for (int u = 0; u < kAhead; ++u) {
        const uint64_t e = g0 + (uint64_t)u * kThreads + tid;
        xs[u] = ss_event_t{0xFFFFFFFFu, 0, 0};
        before0[u] = 0;
        if (e < cnt) {
          xs[u] = L[e];
          if (lane == 0 && e > 0) before0[u] = L[e - 1].op_idx;
        }
      }
#pragma unroll
      for (int u = 0; u < kAhead; ++u) {
        const uint64_t e0 = g0 + (uint64_t)u * kThreads;
        if (e0 >= cnt) break;                                            // uniform: shuffles inside
        const uint64_t e = e0 + tid;
        const bool in = e < cnt;
        const ss_event_t x = xs[u];
        const bool live = in && x.op_idx < n;
        if (in && !live) bad |= 1u;
        uint32_t prev = (uint32_t)__shfl_up((int)x.op_idx, 1, 64);
        if (lane == 0) prev = before0[u];
        if (in && e > 0 && prev > x.op_idx) bad |= 2u;
        const bool head = lane == 0 || prev != x.op_idx;
        const bool is_pos = x.delta >= 0;
        const uint64_t H = __ballot(head);
        const uint64_t P = __ballot(live && is_pos), N = __ballot(live && !is_pos);
        // inclusive wavefront prefix sums of the positive and of the negative deltas
        int64_t ip = live && is_pos ? x.delta : 0, ineg = live && !is_pos ? x.delta : 0;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
          const int64_t op_ = shfl_up_i64(ip, d), on_ = shfl_up_i64(ineg, d);
          if (lane >= d) { ip += op_; ineg += on_; }
        }
        const uint64_t later_heads = H & ~below & ~(1ull << lane);
        const int end = later_heads ? __ffsll((unsigned long long)later_heads) - 1 : 64;   // one past the run's last lane
        int64_t bp = shfl_up_i64(ip, 1), bn = shfl_up_i64(ineg, 1);      // totals before this lane
        if (lane == 0) { bp = 0; bn = 0; }
        const int last = end - 1;
        const int64_t ep = (int64_t)(((uint64_t)(uint32_t)__shfl((int)(uint32_t)((uint64_t)ip >> 32), last, 64) << 32) |
                                     (uint32_t)__shfl((int)(uint32_t)(uint64_t)ip, last, 64));
        const int64_t en = (int64_t)(((uint64_t)(uint32_t)__shfl((int)(uint32_t)((uint64_t)ineg >> 32), last, 64) << 32) |
                                     (uint32_t)__shfl((int)(uint32_t)(uint64_t)ineg, last, 64));
        if (head && live) {
          const uint64_t run = (end == 64 ? ~0ull : ((1ull << end) - 1)) & ~below;
          const uint32_t np = (uint32_t)__popcll(P & run), nn = (uint32_t)__popcll(N & run);
          if (np) {
            add_i64(a.csum + (uint64_t)cpos * n + x.op_idx, ep - bp);
            atomicAdd(a.ccnt + (uint64_t)cpos * n + x.op_idx, np);
          }
          if (nn) {
            add_i64(a.csum + (uint64_t)cneg * n + x.op_idx, en - bn);
            atomicAdd(a.ccnt + (uint64_t)cneg * n + x.op_idx, nn);
          }
        }
      }
    }
  }
  return bad;
}

// `gathered`: phases 0 and 1 have been done by launches before this one (a.flags holds their flags)
__device__ __forceinline__ void scan_body(const ScanArgs &a, bool gathered) {
  __shared__ int64_t wsum[kWaves];
  __shared__ int64_t red_val[kWaves];
  __shared__ uint32_t red_idx[kWaves];
  __shared__ uint32_t red_cnt[kWaves];
  __shared__ uint32_t s_flags;
  const uint32_t tid = threadIdx.x;
  const uint32_t n = a.n_ops;
  if (tid == 0) s_flags = gathered ? *a.flags : 0;
  if (!gathered) {
    // phase 0: clear the per-operator accumulators
    for (uint64_t i = tid; i < 4ull * n; i += kThreads) {
      a.csum[i] = 0;
      a.ccnt[i] = 0;
    }
    __threadfence();
    __syncthreads();
    const uint32_t bad = gather_events(a, 0, 1);
    if (bad) atomicOr(&s_flags, bad);
  }
  __threadfence();
  __syncthreads();
  const uint32_t flags = s_flags;
  if (flags & 1u) {                       // an operator index out of range: nothing else is meaningful
    if (tid == 0) {
      *a.flags = flags;
      if (a.res_flags) {
        ss_scan_result_t r = {a.base, a.base, -1, 0, 0, flags};
        *a.res = r;
      }
    }
    return;
  }

  // phase 2: prefix scan over operators
  int64_t carry = 0;                      // deltas of all operators before this chunk
  uint32_t carry_cnt = 0;
  int64_t best = INT64_MIN;
  uint32_t best_t = 0xFFFFFFFFu, over = 0;
  for (uint32_t c0 = 0; c0 < n; c0 += kThreads) {
    const uint32_t t = c0 + tid;
    int64_t pos = 0, net = 0;
    uint32_t cnt = 0;
    if (t < n) {
      const int64_t s0 = a.csum[t], s1 = a.csum[(uint64_t)n + t], s2 = a.csum[2ull * n + t],
                    s3 = a.csum[3ull * n + t];
      pos = s0 + s1;
      net = pos + s2 + s3;
      cnt = a.ccnt[t] + a.ccnt[(uint64_t)n + t] + a.ccnt[2ull * n + t] + a.ccnt[3ull * n + t];
    }
    int64_t tot, tot_cnt;
    const int64_t inc = block_scan_i64(net, wsum, tot);
    const int64_t inc_cnt = block_scan_i64((int64_t)cnt, wsum, tot_cnt);
    if (t < n) {
      const int64_t entry = carry + inc - net;            // held on entry to t (without base)
      const int64_t p = a.base + entry + pos;             // entry + everything t allocates
      a.before[t] = entry;
      a.evstart[t] = carry_cnt + (uint32_t)(inc_cnt - cnt);
      if (a.per_op) a.per_op[t] = p;
      const int64_t ex = p > a.budget ? p - a.budget : 0;
      if (a.mre) a.mre[t] = ex;
      over += ex > 0;
      if (p > best) { best = p; best_t = t; }             // ascending t per lane: first maximum kept
    }
    carry += tot;
    carry_cnt += (uint32_t)tot_cnt;
  }
  // workgroup reduction: maximum, its first operator, number of over-budget operators
  {
    const int lane = tid & 63, w = tid >> 6;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      const int64_t ob = (int64_t)(((uint64_t)(uint32_t)__shfl_down((int)(uint32_t)((uint64_t)best >> 32), d, 64) << 32) |
                                   (uint32_t)__shfl_down((int)(uint32_t)(uint64_t)best, d, 64));
      const uint32_t ot = (uint32_t)__shfl_down((int)best_t, d, 64);
      const uint32_t oo = (uint32_t)__shfl_down((int)over, d, 64);
      if (lane + d < 64) {
        if (ob > best || (ob == best && ot < best_t)) { best = ob; best_t = ot; }
        over += oo;
      }
    }
    if (lane == 0) { red_val[w] = best; red_idx[w] = best_t; red_cnt[w] = over; }
    __syncthreads();
    if (tid == 0) {
      int64_t b = INT64_MIN; uint32_t bt = 0xFFFFFFFFu, oc = 0;
      for (int i = 0; i < kWaves; ++i) {
        if (red_val[i] > b || (red_val[i] == b && red_idx[i] < bt)) { b = red_val[i]; bt = red_idx[i]; }
        oc += red_cnt[i];
      }
      ss_scan_result_t r;
      r.peak = n ? b : a.base;
      r.final_total = a.base + carry;
      r.argpeak_op = n ? (int32_t)bt : -1;
      r.n_over = oc;
      r.sorted = (flags & 2u) ? 0u : 1u;
      r.reserved = a.res_flags ? flags : 0;
      *a.res = r;
      *a.flags = flags;
    }
  }
  if (!a.want_timeline || (flags & 2u)) return;
  __threadfence();
  __syncthreads();

  // phase 3a: running sum and count of each event's own class along its list; remember
  // them at the first event of every operator
  for (int list = 0; list < 2; ++list) {
    const ss_event_t *L = list ? a.pev : a.ev;
    const uint64_t cnt = list ? a.n_pe : a.n_ev;
    const uint64_t out0 = list ? a.n_ev : 0;
    const int cpos = list ? 0 : 1, cneg = list ? 3 : 2;
    int64_t cs_pos = 0, cs_neg = 0, cc_pos = 0, cc_neg = 0;      // carries
    for (uint64_t e0 = 0; e0 < cnt; e0 += kThreads) {
      const uint64_t e = e0 + tid;
      ss_event_t x = {0, 0, 0};
      bool live = e < cnt, is_pos = false;
      if (live) { x = L[e]; is_pos = x.delta >= 0; }
      int64_t t_sp, t_sn, t_cp, t_cn;
      const int64_t i_sp = block_scan_i64(live && is_pos ? x.delta : 0, wsum, t_sp);
      const int64_t i_sn = block_scan_i64(live && !is_pos ? x.delta : 0, wsum, t_sn);
      const int64_t i_cp = block_scan_i64(live && is_pos ? 1 : 0, wsum, t_cp);
      const int64_t i_cn = block_scan_i64(live && !is_pos ? 1 : 0, wsum, t_cn);
      if (live) {
        // exclusive values at e
        const int64_t xsp = cs_pos + i_sp - (is_pos ? x.delta : 0);
        const int64_t xsn = cs_neg + i_sn - (!is_pos ? x.delta : 0);
        const uint32_t xcp = (uint32_t)(cc_pos + i_cp - (is_pos ? 1 : 0));
        const uint32_t xcn = (uint32_t)(cc_neg + i_cn - (!is_pos ? 1 : 0));
        a.sumx[out0 + e] = is_pos ? xsp : xsn;
        a.cntx[out0 + e] = is_pos ? xcp : xcn;
        if (e == 0 || L[e - 1].op_idx != x.op_idx) {
          a.segsum[(uint64_t)cpos * n + x.op_idx] = xsp;
          a.segsum[(uint64_t)cneg * n + x.op_idx] = xsn;
          a.segcnt[(uint64_t)cpos * n + x.op_idx] = xcp;
          a.segcnt[(uint64_t)cneg * n + x.op_idx] = xcn;
        }
      }
      cs_pos += t_sp; cs_neg += t_sn; cc_pos += t_cp; cc_neg += t_cn;
    }
  }
  __threadfence();
  __syncthreads();

  // phase 3b: canonical position and running total of every event
  for (int list = 0; list < 2; ++list) {
    const ss_event_t *L = list ? a.pev : a.ev;
    const uint64_t cnt = list ? a.n_pe : a.n_ev;
    const uint64_t out0 = list ? a.n_ev : 0;
    for (uint64_t e = tid; e < cnt; e += kThreads) {
      const ss_event_t x = L[e];
      const uint32_t t = x.op_idx;
      const int c = event_class(list != 0, x.delta);
      uint32_t q = a.evstart[t];
      int64_t v = a.base + a.before[t];
      for (int c2 = 0; c2 < c; ++c2) {
        q += a.ccnt[(uint64_t)c2 * n + t];
        v += a.csum[(uint64_t)c2 * n + t];
      }
      q += a.cntx[out0 + e] - a.segcnt[(uint64_t)c * n + t];
      v += a.sumx[out0 + e] - a.segsum[(uint64_t)c * n + t] + x.delta;
      a.timeline[q] = v;
    }
  }
}

__global__ __launch_bounds__(kThreads) void ss_scan_kernel(ScanArgs a) { scan_body(a, false); }

// one workgroup per scan: candidate policies against the same trace in a single launch
__global__ __launch_bounds__(kThreads) void ss_scan_batch_kernel(const ScanArgs *__restrict__ args) {
  const ScanArgs a = args[blockIdx.x];
  scan_body(a, false);
}

// Long traces: the gather is the part that grows with the number of events (one workgroup takes 1.6 us per
// thousand events), and it is the part that splits: the accumulators are cleared by one launch, gathered
// into by a launch of many workgroups, and the rest (the scan over the operators, the timeline) runs in one
// workgroup as before.
__global__ __launch_bounds__(kThreads) void ss_scan_clear_kernel(ScanArgs a) {
  const uint64_t total = 4ull * a.n_ops;
  for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (uint64_t)gridDim.x * kThreads) {
    a.csum[i] = 0;
    a.ccnt[i] = 0;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) *a.flags = 0;
}

__global__ __launch_bounds__(kThreads) void ss_scan_gather_kernel(ScanArgs a) {
  const uint32_t bad = gather_events(a, blockIdx.x, gridDim.x);
  if (bad) atomicOr(a.flags, bad);
}

__global__ __launch_bounds__(kThreads) void ss_scan_finish_kernel(ScanArgs a) { scan_body(a, true); }

constexpr uint64_t kSplitFromEvents = 32768;     // below this one workgroup is as fast as three launches

void launch_scan(hipStream_t s, const ScanArgs &a) {
  const uint64_t E = a.n_ev + a.n_pe;
  if (E < kSplitFromEvents) {
    hipLaunchKernelGGL(ss_scan_kernel, dim3(1), dim3(kThreads), 0, s, a);
    return;
  }
  const uint64_t per_wg = 4ull * kThreads;         // one pass of the gather loop per workgroup
  const uint32_t g_clear = (uint32_t)std::min<uint64_t>(256, (4ull * a.n_ops + kThreads - 1) / kThreads + 1);
  const uint32_t g_gather = (uint32_t)std::min<uint64_t>(512, (std::max(a.n_ev, a.n_pe) + per_wg - 1) / per_wg);
  hipLaunchKernelGGL(ss_scan_clear_kernel, dim3(g_clear), dim3(kThreads), 0, s, a);
  hipLaunchKernelGGL(ss_scan_gather_kernel, dim3(g_gather), dim3(kThreads), 0, s, a);
  hipLaunchKernelGGL(ss_scan_finish_kernel, dim3(1), dim3(kThreads), 0, s, a);
}

}  // namespace

// ---- the scan for callers that cannot allocate ------------------------------------------------
//
// Same kernel, but its scratch (per-operator class sums and counts, entry totals, event
// positions, per-event class prefixes) lives in a static device array instead of memory the
// library allocates, and inputs and outputs are the caller's device arrays: the call only
// enqueues the scan's kernels (one, or three for a long trace) on the caller's stream.

constexpr uint32_t kStaticMaxOps = 65536;
constexpr uint64_t kStaticMaxEvents = 262144;
constexpr size_t kStaticBytes =
    2 * (4ull * kStaticMaxOps * 8)        // csum, segsum
    + 1ull * kStaticMaxOps * 8            // before
    + 2 * (4ull * kStaticMaxOps * 4)      // ccnt, segcnt
    + 1ull * kStaticMaxOps * 4            // evstart
    + kStaticMaxEvents * 8                // sumx
    + kStaticMaxEvents * 4                // cntx
    + 256;                                // flags
static __device__ __align__(256) uint8_t scratch[kStaticBytes];

// Address of `scratch` on each device (the name itself is only a host-side handle): resolved once
// per device, with that device current.
constexpr int kMaxDevices = 64;
static uint8_t *g_scratch_ptr[kMaxDevices];

static int static_scratch_ptr(int device, uint8_t **out, hipError_t *err) {
  *err = hipSuccess;
  if (device < 0 || device >= kMaxDevices) return SS_E_INVAL;
  if (!g_scratch_ptr[device]) {
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      *err = e;
      return SS_E_HIP;
    }
    g_scratch_ptr[device] = (uint8_t *)p;
  }
  *out = g_scratch_ptr[device];
  return SS_OK;
}

int ss_scan_static_init(ss_ctx *ctx) {
  uint8_t *p;
  hipError_t e;
  const int rc = static_scratch_ptr(ctx->device, &p, &e);
  if (rc == SS_E_HIP) SS_HIP(e);
  return rc;
}

extern "C" int ss_timeline_scan_static(ss_ctx *ctx, void *stream, const ss_event_t *d_ev, uint64_t n_ev,
                                       const ss_event_t *d_pev, uint64_t n_pe, uint32_t n_ops, int64_t base,
                                       int64_t budget, int64_t *d_timeline, int64_t *d_per_op, int64_t *d_mre,
                                       ss_scan_result_t *d_res) {
  if (!ctx || !d_res || (n_ev && !d_ev) || (n_pe && !d_pev)) return SS_E_INVAL;
  if (n_ops > kStaticMaxOps || n_ev > kStaticMaxEvents || n_pe > kStaticMaxEvents || n_ev + n_pe > kStaticMaxEvents)
    return SS_E_CAPACITY;
  int dev = -1;
  SS_HIP(hipGetDevice(&dev));
  if (dev != ctx->device) return SS_E_STATE;          // the context's copy of the array is on its own device
  uint8_t *d = nullptr;
  hipError_t e;
  const int rc = static_scratch_ptr(dev, &d, &e);
  if (rc == SS_E_HIP) SS_HIP(e);
  if (rc != SS_OK) return rc;
  const uint64_t n = kStaticMaxOps, E = kStaticMaxEvents;    // fixed layout: every piece at its maximum
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += bytes; return o; };
  ScanArgs a;
  a.ev = d_ev; a.n_ev = n_ev;
  a.pev = d_pev; a.n_pe = n_pe;
  a.n_ops = n_ops; a.want_timeline = d_timeline != nullptr;
  a.base = base; a.budget = budget;
  a.csum = (int64_t *)(d + take(4 * n * 8));
  a.segsum = (int64_t *)(d + take(4 * n * 8));
  a.before = (int64_t *)(d + take(n * 8));
  a.sumx = (int64_t *)(d + take(E * 8));
  a.ccnt = (uint32_t *)(d + take(4 * n * 4));
  a.segcnt = (uint32_t *)(d + take(4 * n * 4));
  a.evstart = (uint32_t *)(d + take(n * 4));
  a.cntx = (uint32_t *)(d + take(E * 4));
  a.flags = (uint32_t *)(d + take(256));
  a.per_op = d_per_op; a.mre = d_mre; a.timeline = d_timeline;
  a.res = d_res;
  a.res_flags = 1;
  launch_scan((hipStream_t)stream, a);
  SS_HIP(hipGetLastError());
  return SS_OK;
}

extern "C" int ss_timeline_scan_batch(ss_ctx *ctx, const ss_event_t *ev, uint64_t n_ev, const ss_event_t *pev,
                                      const uint64_t *pe_start, uint32_t k, uint32_t n_ops, int64_t base,
                                      int64_t budget, int64_t *per_op, ss_scan_result_t *res) {
  return ss_guard([&]() -> int {
    if (!ctx || (k && (!res || !pe_start)) || (n_ev && !ev)) return SS_E_INVAL;
    if (k == 0) return SS_OK;
    if (k > 4096 || n_ops > (1u << 23)) return SS_E_INVAL;
    const uint64_t n_pe = pe_start[k];
    for (uint32_t c = 0; c < k; ++c)
      if (pe_start[c] > pe_start[c + 1]) return SS_E_INVAL;
    if (pe_start[0] != 0 || (n_pe && !pev) || n_ev + n_pe >= (1ull << 31)) return SS_E_INVAL;
    const uint64_t n = n_ops;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += ss_align_up(bytes, 256); return o; };
    const size_t o_ev = take(n_ev * sizeof(ss_event_t)), o_pev = take(n_pe * sizeof(ss_event_t));
    const size_t o_args = take((size_t)k * sizeof(ScanArgs)), o_res = take((size_t)k * sizeof(ss_scan_result_t));
    const size_t o_flags = take((size_t)k * 4);
    const size_t per_scan = ss_align_up(4 * n * 8, 256) + 3 * ss_align_up(n * 8, 256) + ss_align_up(4 * n * 4, 256) +
                            ss_align_up(n * 4, 256);
    const size_t o_work = take((size_t)k * per_scan);
    const size_t host_bytes = (size_t)k * (sizeof(ScanArgs) + sizeof(ss_scan_result_t) + 4) + 1024;
    int rc = ss_scratch_reserve(ctx, off, host_bytes);
    if (rc != SS_OK) return rc;
    uint8_t *d = (uint8_t *)ctx->d_scratch, *h = (uint8_t *)ctx->h_scratch;
    hipStream_t s = ctx->s_aux;
    if (n_ev) SS_HIP(hipMemcpyAsync(d + o_ev, ev, n_ev * sizeof(ss_event_t), hipMemcpyHostToDevice, s));
    if (n_pe) SS_HIP(hipMemcpyAsync(d + o_pev, pev, n_pe * sizeof(ss_event_t), hipMemcpyHostToDevice, s));
    ScanArgs *ha = (ScanArgs *)h;                       // pinned: argument blocks, then results and flags
    for (uint32_t c = 0; c < k; ++c) {
      uint8_t *w = d + o_work + (size_t)c * per_scan;
      size_t wo = 0;
      auto wtake = [&](size_t bytes) { uint8_t *p = w + wo; wo += ss_align_up(bytes, 256); return p; };
      ScanArgs a;
      std::memset(&a, 0, sizeof(a));
      a.ev = (const ss_event_t *)(d + o_ev); a.n_ev = n_ev;
      a.pev = (const ss_event_t *)(d + o_pev) + pe_start[c]; a.n_pe = pe_start[c + 1] - pe_start[c];
      a.n_ops = n_ops; a.want_timeline = 0;
      a.base = base; a.budget = budget;
      a.csum = (int64_t *)wtake(4 * n * 8);
      a.before = (int64_t *)wtake(n * 8);
      a.per_op = (int64_t *)wtake(n * 8);
      a.mre = (int64_t *)wtake(n * 8);
      a.ccnt = (uint32_t *)wtake(4 * n * 4);
      a.evstart = (uint32_t *)wtake(n * 4);
      a.res = (ss_scan_result_t *)(d + o_res) + c;
      a.flags = (uint32_t *)(d + o_flags) + c;
      ha[c] = a;
    }
    SS_HIP(hipMemcpyAsync(d + o_args, ha, (size_t)k * sizeof(ScanArgs), hipMemcpyHostToDevice, s));
    hipLaunchKernelGGL(ss_scan_batch_kernel, dim3(k), dim3(kThreads), 0, s, (const ScanArgs *)(d + o_args));
    SS_HIP(hipGetLastError());
    uint8_t *hres = h + ss_align_up((size_t)k * sizeof(ScanArgs), 256);
    uint8_t *hflags = hres + (size_t)k * sizeof(ss_scan_result_t);
    SS_HIP(hipMemcpyAsync(hres, d + o_res, (size_t)k * sizeof(ss_scan_result_t), hipMemcpyDeviceToHost, s));
    SS_HIP(hipMemcpyAsync(hflags, d + o_flags, (size_t)k * 4, hipMemcpyDeviceToHost, s));
    SS_HIP(hipStreamSynchronize(s));
    for (uint32_t c = 0; c < k; ++c) {
      uint32_t fl;
      std::memcpy(&fl, hflags + 4 * (size_t)c, 4);
      if (fl & 1u) return SS_E_INVAL;
    }
    std::memcpy(res, hres, (size_t)k * sizeof(ss_scan_result_t));
    if (per_op && n) {
      for (uint32_t c = 0; c < k; ++c)
        SS_HIP(hipMemcpyAsync(per_op + (size_t)c * n, ha[c].per_op, n * 8, hipMemcpyDeviceToHost, s));
      SS_HIP(hipStreamSynchronize(s));
    }
    return SS_OK;
  });
}

extern "C" int ss_timeline_scan(ss_ctx *ctx, const ss_event_t *ev, uint64_t n_ev, const ss_event_t *pev,
                                uint64_t n_pe, uint32_t n_ops, int64_t base, int64_t budget,
                                int64_t *timeline, int64_t *per_op, int64_t *mre, ss_scan_result_t *res) {
  return ss_guard([&]() -> int {
    if (!ctx || !res || (n_ev && !ev) || (n_pe && !pev)) return SS_E_INVAL;
    if (n_ops > (1u << 23) || n_ev + n_pe >= (1ull << 31)) return SS_E_INVAL;
    const uint64_t E = n_ev + n_pe;
    const uint64_t n = n_ops;
    // device layout (8-byte aligned pieces first)
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += ss_align_up(bytes, 256); return o; };
    const size_t o_ev = take(n_ev * sizeof(ss_event_t)), o_pev = take(n_pe * sizeof(ss_event_t));
    const size_t o_csum = take(4 * n * 8), o_before = take(n * 8), o_segsum = take(4 * n * 8);
    const size_t o_sumx = take(E * 8), o_perop = take(n * 8), o_mre = take(n * 8), o_tl = take(E * 8);
    const size_t o_ccnt = take(4 * n * 4), o_evstart = take(n * 4), o_segcnt = take(4 * n * 4);
    const size_t o_cntx = take(E * 4), o_res = take(sizeof(ss_scan_result_t)), o_flags = take(4);
    int rc = ss_scratch_reserve(ctx, off, 512);
    if (rc != SS_OK) return rc;
    uint8_t *d = (uint8_t *)ctx->d_scratch;
    hipStream_t s = ctx->s_aux;
    if (n_ev) SS_HIP(hipMemcpyAsync(d + o_ev, ev, n_ev * sizeof(ss_event_t), hipMemcpyHostToDevice, s));
    if (n_pe) SS_HIP(hipMemcpyAsync(d + o_pev, pev, n_pe * sizeof(ss_event_t), hipMemcpyHostToDevice, s));
    ScanArgs a;
    a.res_flags = 0;
    a.ev = (const ss_event_t *)(d + o_ev); a.n_ev = n_ev;
    a.pev = (const ss_event_t *)(d + o_pev); a.n_pe = n_pe;
    a.n_ops = n_ops; a.want_timeline = timeline != nullptr;
    a.base = base; a.budget = budget;
    a.csum = (int64_t *)(d + o_csum); a.ccnt = (uint32_t *)(d + o_ccnt);
    a.before = (int64_t *)(d + o_before); a.evstart = (uint32_t *)(d + o_evstart);
    a.segsum = (int64_t *)(d + o_segsum); a.segcnt = (uint32_t *)(d + o_segcnt);
    a.sumx = (int64_t *)(d + o_sumx); a.cntx = (uint32_t *)(d + o_cntx);
    a.per_op = (int64_t *)(d + o_perop); a.mre = (int64_t *)(d + o_mre);
    a.timeline = (int64_t *)(d + o_tl);
    a.res = (ss_scan_result_t *)(d + o_res); a.flags = (uint32_t *)(d + o_flags);
    launch_scan(s, a);
    SS_HIP(hipGetLastError());
    uint8_t *h = (uint8_t *)ctx->h_scratch;            // pinned: result + flags
    SS_HIP(hipMemcpyAsync(h, d + o_res, sizeof(ss_scan_result_t), hipMemcpyDeviceToHost, s));
    SS_HIP(hipMemcpyAsync(h + 256, d + o_flags, 4, hipMemcpyDeviceToHost, s));
    SS_HIP(hipStreamSynchronize(s));
    uint32_t flags;
    std::memcpy(&flags, h + 256, 4);
    if (flags & 1u) return SS_E_INVAL;
    std::memcpy(res, h, sizeof(*res));
    if (per_op && n) SS_HIP(hipMemcpyAsync(per_op, d + o_perop, n * 8, hipMemcpyDeviceToHost, s));
    if (mre && n) SS_HIP(hipMemcpyAsync(mre, d + o_mre, n * 8, hipMemcpyDeviceToHost, s));
    const bool tl_ok = timeline && !(flags & 2u);
    if (tl_ok && E) SS_HIP(hipMemcpyAsync(timeline, d + o_tl, E * 8, hipMemcpyDeviceToHost, s));
    SS_HIP(hipStreamSynchronize(s));
    if (timeline && !tl_ok) return SS_E_ORDER;
    return SS_OK;
  });
}
