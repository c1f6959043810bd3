// Operator-sequence matcher on the GPU.
//
// (i) Similarity of two integer operator sequences and the stage machine of Algo. 1
//     (Sec. 3 of the SmartSwap paper): length within 5 %, cosine above 95 %.  The three
//     integer sums of the cosine are reduced on the GPU; the threshold is decided exactly
//     on the host in 128-bit integer arithmetic.
// (ii) Re-anchoring of policy items in the current sequence (Sec. 5.1: multi-feature
//     matching on operator name, call stack and data type with integer comparisons
//     only).  One wavefront serves one anchor: it counts, with per-lane compares and a
//     wavefront reduction, how many earlier operators of the reference share the anchor's
//     key at each of three relaxation levels, then walks the current sequence 64
//     operators at a time, using ballots and population counts to find the operator of
//     that ordinal.
#include <cstring>

#include "ss_internal.h"

namespace {

constexpr uint32_t kTokenLimit = 1u << 18;
constexpr uint32_t kLenLimit = 1u << 23;

__device__ inline uint64_t wave_sum_u64(uint64_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)v, d, 64);
    uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(v >> 32), d, 64);
    v += ((uint64_t)hi << 32) | lo;
  }
  return v;
}

// sums[0] = dot, sums[1] = na (current), sums[2] = nb (reference), flags bit 0: token too large
__global__ __launch_bounds__(256) void ss_cosine_kernel(const ss_op_t *__restrict__ ref, uint32_t n,
                                                        const ss_op_t *__restrict__ cur, uint32_t m,
                                                        unsigned long long *sums, uint32_t *flags) {
  __shared__ uint64_t part[3][4];
  const uint32_t len = n > m ? n : m;
  uint64_t dot = 0, na = 0, nb = 0;
  uint32_t bad = 0;
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < len; i += gridDim.x * blockDim.x) {
    const uint64_t a = i < m ? cur[i].op_token : 0;     // the shorter sequence is padded with token 0
    const uint64_t b = i < n ? ref[i].op_token : 0;
    if (a >= kTokenLimit || b >= kTokenLimit) bad = 1;
    dot += a * b;
    na += a * a;
    nb += b * b;
  }
  dot = wave_sum_u64(dot); na = wave_sum_u64(na); nb = wave_sum_u64(nb);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (lane == 0) { part[0][w] = dot; part[1][w] = na; part[2][w] = nb; }
  __syncthreads();
  if (threadIdx.x < 3) {
    uint64_t s = part[threadIdx.x][0] + part[threadIdx.x][1] + part[threadIdx.x][2] + part[threadIdx.x][3];
    if (s) atomicAdd(sums + threadIdx.x, (unsigned long long)s);
  }
  if (bad) atomicOr(flags, 1u);
}

// occurrence counts per token of both sequences (token 0 never counts)
__global__ __launch_bounds__(256) void ss_histogram_kernel(const ss_op_t *__restrict__ ref, uint32_t n,
                                                           const ss_op_t *__restrict__ cur, uint32_t m,
                                                           uint32_t *h_ref, uint32_t *h_cur, uint32_t *flags) {
  const uint32_t len = n > m ? n : m;
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < len; i += gridDim.x * blockDim.x) {
    if (i < m) {
      const uint32_t a = cur[i].op_token;
      if (a >= kTokenLimit) atomicOr(flags, 1u); else if (a) atomicAdd(h_cur + a, 1u);
    }
    if (i < n) {
      const uint32_t b = ref[i].op_token;
      if (b >= kTokenLimit) atomicOr(flags, 1u); else if (b) atomicAdd(h_ref + b, 1u);
    }
  }
}

__global__ __launch_bounds__(256) void ss_histdot_kernel(const uint32_t *__restrict__ h_ref,
                                                         const uint32_t *__restrict__ h_cur, uint32_t vocab,
                                                         unsigned long long *sums) {
  __shared__ uint64_t part[3][4];
  uint64_t dot = 0, na = 0, nb = 0;
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < vocab; i += gridDim.x * blockDim.x) {
    const uint64_t a = h_cur[i], b = h_ref[i];
    dot += a * b; na += a * a; nb += b * b;
  }
  dot = wave_sum_u64(dot); na = wave_sum_u64(na); nb = wave_sum_u64(nb);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (lane == 0) { part[0][w] = dot; part[1][w] = na; part[2][w] = nb; }
  __syncthreads();
  if (threadIdx.x < 3) {
    uint64_t s = part[threadIdx.x][0] + part[threadIdx.x][1] + part[threadIdx.x][2] + part[threadIdx.x][3];
    if (s) atomicAdd(sums + threadIdx.x, (unsigned long long)s);
  }
}

__device__ inline uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += (uint32_t)__shfl_xor((int)v, d, 64);
  return v;
}

// Lane index of the bit of `mask` that has exactly `need` set bits below it.
__device__ inline int nth_set_bit(uint64_t mask, uint32_t need, int lane) {
  const uint64_t below = lane ? (mask & (~0ull >> (64 - lane))) : 0ull;
  const bool mine = ((mask >> lane) & 1ull) && (uint32_t)__popcll(below) == need;
  const uint64_t sel = __ballot(mine);
  return __ffsll((long long)sel) - 1;
}

// One wavefront per anchor.  land[a] = operator index in cur (or -1), lvl[a] = level (or 255).
__global__ __launch_bounds__(256) void ss_anchor_kernel(const ss_op_t *__restrict__ ref, uint32_t n,
                                                        const ss_op_t *__restrict__ cur, uint32_t m,
                                                        const ss_anchor_t *__restrict__ anchors, uint32_t k,
                                                        int32_t *land, uint8_t *lvl) {
  const int lane = threadIdx.x & 63;
  const uint32_t a = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  if (a >= k) return;                                   // uniform per wavefront
  const uint32_t i = anchors[a].ref_op, s = anchors[a].out_slot;
  int32_t result = -1;
  uint8_t level = 255;
  if (i < n && ref[i].op_token != 0) {
    const ss_op_t R = ref[i];
    // ordinal of ref[i] among the earlier operators with the same key, per level
    uint32_t r0 = 0, r1 = 0, r2 = 0;
    for (uint32_t j = lane; j < i; j += 64) {
      const ss_op_t o = ref[j];
      const bool e2 = o.op_token == R.op_token;
      const bool e1 = e2 && o.sig == R.sig;
      const bool e0 = e1 && o.stack_hash == R.stack_hash;
      r2 += e2; r1 += e1; r0 += e0;
    }
    r0 = wave_sum_u32(r0); r1 = wave_sum_u32(r1); r2 = wave_sum_u32(r2);
    // operator of that ordinal in cur, per level
    int32_t f0 = -1, f1 = -1, f2 = -1;
    uint32_t c0 = 0, c1 = 0, c2 = 0;                    // matches seen so far (uniform)
    for (uint32_t base = 0; base < m; base += 64) {
      const uint32_t j = base + lane;
      bool e0 = false, e1 = false, e2 = false;
      if (j < m) {
        const ss_op_t o = cur[j];
        e2 = o.op_token == R.op_token;
        e1 = e2 && o.sig == R.sig;
        e0 = e1 && o.stack_hash == R.stack_hash;
      }
      const uint64_t b0 = __ballot(e0), b1 = __ballot(e1), b2 = __ballot(e2);
      if (f0 < 0) { const uint32_t pc = __popcll(b0); if (c0 + pc > r0) f0 = (int32_t)base + nth_set_bit(b0, r0 - c0, lane); else c0 += pc; }
      if (f1 < 0) { const uint32_t pc = __popcll(b1); if (c1 + pc > r1) f1 = (int32_t)base + nth_set_bit(b1, r1 - c1, lane); else c1 += pc; }
      if (f2 < 0) { const uint32_t pc = __popcll(b2); if (c2 + pc > r2) f2 = (int32_t)base + nth_set_bit(b2, r2 - c2, lane); else c2 += pc; }
      if (f0 >= 0 && f1 >= 0 && f2 >= 0) break;
    }
    const int32_t f[3] = {f0, f1, f2};
    const uint32_t want = R.sig & 0xFFu;
#pragma unroll
    for (int L = 0; L < 3; ++L) {
      if (result >= 0 || f[L] < 0) continue;
      const ss_op_t o = cur[f[L]];
      if (s < o.n_out && (o.sig & 0xFFu) == want) { result = f[L]; level = (uint8_t)L; }
    }
  }
  if (lane == 0) { land[a] = result; lvl[a] = level; }
}

// Among anchors landing on the same (operator, slot) only the lowest anchor index keeps it.
// Two passes over an open-addressing table of at least 2k slots keyed by (operator, slot): every
// landed anchor finds or claims its key's slot (compare-and-swap, linear probing) and lowers the
// slot's owner to its own index (integer minimum: any order, same result); then an anchor keeps its
// landing exactly if it owns its slot.  Linear in k (20,000 anchors: all earlier anchors compared one
// by one took 2 ms).
constexpr unsigned long long kEmptyKey = ~0ull;

__global__ __launch_bounds__(256) void ss_claim_kernel(const ss_anchor_t *__restrict__ anchors, uint32_t k,
                                                       const int32_t *__restrict__ land,
                                                       unsigned long long *keys, uint32_t *owner,
                                                       uint32_t *__restrict__ slot_of, uint32_t mask,
                                                       uint32_t shift) {
  const uint32_t a = blockIdx.x * blockDim.x + threadIdx.x;
  if (a >= k) return;
  const int32_t j = land[a];
  if (j < 0) return;
  const unsigned long long key = ((unsigned long long)(uint32_t)j << 32) | anchors[a].out_slot;   // j < 2^31: never kEmptyKey
  uint32_t h = (uint32_t)((key * 0x9E3779B97F4A7C15ull) >> shift);
  // at most k distinct keys in more than 2k slots: a free or matching slot is met within mask + 1 probes
  for (uint32_t probe = 0; probe <= mask; ++probe) {
    const unsigned long long seen = atomicCAS(keys + h, kEmptyKey, key);
    if (seen == kEmptyKey || seen == key) {
      atomicMin(owner + h, a);
      slot_of[a] = h;
      return;
    }
    h = (h + 1) & mask;
  }
}

__global__ __launch_bounds__(256) void ss_injective_kernel(uint32_t k, const int32_t *__restrict__ land,
                                                           const uint8_t *__restrict__ lvl,
                                                           const uint32_t *__restrict__ slot_of,
                                                           const uint32_t *__restrict__ owner, int32_t *new_idx,
                                                           uint8_t *level, uint32_t *n_unmatched) {
  const uint32_t a = blockIdx.x * blockDim.x + threadIdx.x;
  bool lost = false;
  if (a < k) {
    int32_t j = land[a];
    uint8_t L = lvl[a];
    if (j >= 0 && owner[slot_of[a]] != a) { j = -1; L = 255; }
    new_idx[a] = j;
    level[a] = L;
    lost = j < 0;
  }
  const uint64_t m = __ballot(lost);
  if ((threadIdx.x & 63) == 0 && m) atomicAdd(n_unmatched, (uint32_t)__popcll(m));
}

}  // namespace

// The stage machine of Algo. 1 as a table: a stage is left for `next` once more than `patience`
// consecutive similar iterations have been counted in it (the count includes the current one), and the
// count starts over if `restart` is set; a stage without a row entry to leave (Stable) only counts.
// Any dissimilar iteration sends every stage back to WarmUp with the count at zero.
struct StagePromotion { bool leaves; uint32_t next; bool restart; };

static void stage_step(ss_ctx *ctx, bool similar) {
  if (!similar) {
    ctx->stage = SS_STAGE_WARMUP;
    ctx->stable_step = 0;
    return;
  }
  const uint32_t patience[3] = {ctx->cfg.stage_m, ctx->cfg.stage_n, 0};
  static const StagePromotion promote[3] = {
      /* WarmUp    */ {true, SS_STAGE_GENPOLICY, true},
      /* GenPolicy */ {true, SS_STAGE_STABLE, false},
      /* Stable    */ {false, SS_STAGE_STABLE, false}};
  const uint32_t from = ctx->stage;
  ctx->stable_step += 1;
  if (from <= SS_STAGE_STABLE && promote[from].leaves && ctx->stable_step > patience[from]) {
    ctx->stage = promote[from].next;
    if (promote[from].restart) ctx->stable_step = 0;
  }
}

extern "C" int ss_match_sequence(ss_ctx *ctx, const ss_op_t *ref, uint32_t n, const ss_op_t *cur, uint32_t m,
                                 const ss_anchor_t *anchors, uint32_t k, uint32_t flags, int32_t *new_idx,
                                 uint8_t *level, ss_match_result_t *res) {
  return ss_guard([&]() -> int {
    if (!ctx || !res || (n && !ref) || (m && !cur)) return SS_E_INVAL;
    if (k && (!anchors || !new_idx || !level)) return SS_E_INVAL;
    if (n > kLenLimit || m > kLenLimit || k > (1u << 24)) return SS_E_INVAL;
    const bool hist = (flags & SS_MATCH_HISTOGRAM) != 0;
    const bool aligned = (flags & SS_MATCH_ALIGN) != 0;
    // verdict, stage machine and counters from the three sums: the same for both routes below
    auto finish = [&](const uint64_t sm[3], uint32_t unm) {
      res->dot = sm[0]; res->na = sm[1]; res->nb = sm[2];
      bool similar;
      if (n == 0 && m == 0) {
        similar = true;
      } else {
        const uint64_t diff = n > m ? n - m : m - n;
        const bool len_ok = 20ull * diff < (uint64_t)n;
        // cos > 0.95  <=>  dot > 0 and 400 dot^2 > 361 na nb; sums < 2^59, so both sides < 2^127
        const unsigned __int128 lhs = (unsigned __int128)400 * sm[0] * sm[0];
        const unsigned __int128 rhs = (unsigned __int128)361 * sm[1] * sm[2];
        similar = len_ok && sm[0] > 0 && lhs > rhs;
      }
      res->similar = similar ? 1u : 0u;
      if (flags & SS_MATCH_STEP_STAGE) stage_step(ctx, similar);
      res->stage = ctx->stage;
      res->stable_step = ctx->stable_step;
      res->n_unmatched = unm;
      for (uint32_t a = 0; a < k; ++a) ctx->stats.match_levels[level[a] <= SS_LEVEL_ALIGN ? level[a] : 4]++;
    };
    // The current sequence IS the reference one (the Stable stage of a fixed operator sequence, Sec. 3):
    // no search is needed.  Every operator is its own counterpart at the strictest level, the three sums
    // coincide, and what remains of the definition (a landing place needs more than out_slot outputs, the
    // lowest anchor index keeps a shared place) is evaluated here on the host in one pass, without a
    // round trip to the GPU.  Results are those of the kernels below on the same input.
    if (!hist && n == m && (n == 0 || std::memcmp(ref, cur, (size_t)n * sizeof(ss_op_t)) == 0)) {
      uint64_t sq = 0;
      for (uint32_t i = 0; i < n; ++i) {
        if (cur[i].op_token >= kTokenLimit) return SS_E_INVAL;
        sq += (uint64_t)cur[i].op_token * cur[i].op_token;
      }
      uint32_t unm = 0;
      if (k) {
        std::unordered_map<uint64_t, uint32_t> first;          // (operator, slot) -> lowest anchor index landing there
        if (!aligned) first.reserve(2 * (size_t)k);
        for (uint32_t a = 0; a < k; ++a) {
          const uint32_t i = anchors[a].ref_op, sl = anchors[a].out_slot;
          const bool lands = i < n && sl < cur[i].n_out && (aligned || cur[i].op_token != 0);
          new_idx[a] = lands ? (int32_t)i : -1;
          level[a] = lands ? (uint8_t)(aligned ? SS_LEVEL_ALIGN : 0) : (uint8_t)255;
          if (lands && !aligned) {
            auto ins = first.emplace(((uint64_t)i << 32) | sl, a);
            if (!ins.second) { new_idx[a] = -1; level[a] = 255; }   // an earlier anchor owns the place
          }
          unm += new_idx[a] < 0;
        }
      }
      const uint64_t sm[3] = {sq, sq, sq};
      finish(sm, unm);
      return SS_OK;
    }
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += ss_align_up(bytes, 256); return o; };
    const size_t o_ref = take((size_t)n * sizeof(ss_op_t)), o_cur = take((size_t)m * sizeof(ss_op_t));
    const size_t o_anc = take((size_t)k * sizeof(ss_anchor_t));
    const size_t o_land = take((size_t)k * 4), o_idx = take((size_t)k * 4);
    const size_t o_lvl = take(k), o_level = take(k);
    const size_t o_small = take(64);                       // 3 x u64 sums, flags, n_unmatched
    const size_t o_hist = take(hist ? 2 * (size_t)kTokenLimit * 4 : 0);
    // table of the injectivity pass: a power of two of at least 2k slots; keys, then owners, back to back
    uint32_t bits = 6;
    while ((1ull << bits) < 2ull * k) ++bits;
    const size_t slots = (size_t)1 << bits;
    const size_t o_keys = take(k ? slots * 8 : 0), o_owner = take(k ? slots * 4 : 0), o_slot = take((size_t)k * 4);
    int rc = ss_scratch_reserve(ctx, off, 512);
    if (rc != SS_OK) return rc;
    uint8_t *d = (uint8_t *)ctx->d_scratch;
    hipStream_t s = ctx->s_aux;
    if (n) SS_HIP(hipMemcpyAsync(d + o_ref, ref, (size_t)n * sizeof(ss_op_t), hipMemcpyHostToDevice, s));
    if (m) SS_HIP(hipMemcpyAsync(d + o_cur, cur, (size_t)m * sizeof(ss_op_t), hipMemcpyHostToDevice, s));
    if (k) SS_HIP(hipMemcpyAsync(d + o_anc, anchors, (size_t)k * sizeof(ss_anchor_t), hipMemcpyHostToDevice, s));
    // zero the small counters (and histograms) with a fill kernel: safe under graph capture too
    ss_launch_fill(s, d + o_small, 64, 0);
    if (hist) ss_launch_fill(s, d + o_hist, 2 * (size_t)kTokenLimit * 4, 0);
    SS_HIP(hipGetLastError());
    unsigned long long *sums = (unsigned long long *)(d + o_small);
    uint32_t *dflags = (uint32_t *)(d + o_small + 32), *d_unm = (uint32_t *)(d + o_small + 40);
    const ss_op_t *dref = (const ss_op_t *)(d + o_ref), *dcur = (const ss_op_t *)(d + o_cur);
    const uint32_t len = n > m ? n : m;
    if (len) {
      uint32_t grid = (len + 255) / 256;
      if (grid > 256) grid = 256;
      if (!hist) {
        hipLaunchKernelGGL(ss_cosine_kernel, dim3(grid), dim3(256), 0, s, dref, n, dcur, m, sums, dflags);
      } else {
        uint32_t *h_ref = (uint32_t *)(d + o_hist), *h_cur = h_ref + kTokenLimit;
        hipLaunchKernelGGL(ss_histogram_kernel, dim3(grid), dim3(256), 0, s, dref, n, dcur, m, h_ref, h_cur, dflags);
        hipLaunchKernelGGL(ss_histdot_kernel, dim3(256), dim3(256), 0, s, h_ref, h_cur, kTokenLimit, sums);
      }
      SS_HIP(hipGetLastError());
    }
    if (k && !aligned) {
      const uint32_t grid = (k + 3) / 4;                    // 4 wavefronts (anchors) per workgroup
      hipLaunchKernelGGL(ss_anchor_kernel, dim3(grid), dim3(256), 0, s, dref, n, dcur, m,
                         (const ss_anchor_t *)(d + o_anc), k, (int32_t *)(d + o_land), d + o_lvl);
      ss_launch_fill(s, d + o_keys, slots * 12, 0xFF);      // every key empty, every owner "nobody" (slots * 8 is a multiple of 256)
      hipLaunchKernelGGL(ss_claim_kernel, dim3((k + 255) / 256), dim3(256), 0, s, (const ss_anchor_t *)(d + o_anc), k,
                         (const int32_t *)(d + o_land), (unsigned long long *)(d + o_keys), (uint32_t *)(d + o_owner),
                         (uint32_t *)(d + o_slot), (uint32_t)(slots - 1), 64u - bits);
      hipLaunchKernelGGL(ss_injective_kernel, dim3((k + 255) / 256), dim3(256), 0, s, k, (const int32_t *)(d + o_land),
                         d + o_lvl, (const uint32_t *)(d + o_slot), (const uint32_t *)(d + o_owner),
                         (int32_t *)(d + o_idx), d + o_level, d_unm);
      SS_HIP(hipGetLastError());
    }
    uint8_t *h = (uint8_t *)ctx->h_scratch;
    SS_HIP(hipMemcpyAsync(h, d + o_small, 64, hipMemcpyDeviceToHost, s));
    if (k && !aligned) {
      SS_HIP(hipMemcpyAsync(new_idx, d + o_idx, (size_t)k * 4, hipMemcpyDeviceToHost, s));
      SS_HIP(hipMemcpyAsync(level, d + o_level, k, hipMemcpyDeviceToHost, s));
    }
    SS_HIP(hipStreamSynchronize(s));
    uint64_t sm[3];
    uint32_t fl, unm;
    std::memcpy(sm, h, 24);
    std::memcpy(&fl, h + 32, 4);
    std::memcpy(&unm, h + 40, 4);
    if (fl & 1u) return SS_E_INVAL;                          // a token beyond 2^18
    uint32_t n_unm = (k && !aligned) ? unm : 0;
    if (k && aligned) {                                      // the scratch is free again: the stream is idle
      std::vector<int32_t> ref_to_cur(n);
      uint32_t lcs = 0;
      rc = ss_align_core(ctx, ref, n, cur, m, ref_to_cur.data(), &lcs, nullptr);
      if (rc != SS_OK) return rc;
      ss_align_anchors(ref, n, cur, ref_to_cur.data(), anchors, k, new_idx, level, &n_unm);
    }
    finish(sm, n_unm);
    return SS_OK;
  });
}
