// Policy application (Sec. 5, first paragraph, of the SmartSwap paper): turn a swap
// policy into the current iteration's action schedule, copy descriptors and the
// policy-induced memory events.  Timing of the release point (Sec. 4.3.2 / 5.2) and of
// the swap-in pre-trigger (Sec. 4.3.1) uses Eq. 3 (T_swap = S / B) at operator
// granularity with one FIFO link per direction; every operator is given the same share
// of the iteration time (Eq. 1 with one operator per group).  Time is counted in link
// bytes: operator t spans [t * bpo, (t + 1) * bpo).
//
// Also here: the longest-idle-first stand-in for the policy generator (Algo. 2), which
// re-times and re-scans (on the GPU) after each added candidate.
#include <algorithm>
#include <cstring>
#include <numeric>

#include "ss_internal.h"

namespace {

struct Live {
  uint32_t a;        // policy index
  uint32_t row;      // row in the tensor table
  uint64_t t_out, t_use, nbytes;
  uint64_t t_free = 0, t_in = 0;
  bool late = false, valid = true, forced = false;
};

typedef unsigned __int128 u128;

// Stable sort of idx by key[idx[i]] ascending: least-significant-digit radix passes of 11 bits,
// skipping digits in which all keys agree.  Every ordering below is "by an operator index, ties by an
// order the list already has", so a stable pass over a pre-ordered list replaces a comparison sort
// (20,000 items: 0.1 ms instead of 2 ms per ordering).
template <class K>
void stable_sort_by(std::vector<uint32_t> &idx, const std::vector<K> &key, std::vector<uint32_t> &tmp) {
  const size_t n = idx.size();
  if (n < 2) return;
  K differ = 0;
  for (size_t i = 1; i < n; ++i) differ |= key[idx[i]] ^ key[idx[0]];
  tmp.resize(n);
  for (unsigned shift = 0; shift < 8 * sizeof(K); shift += 11) {
    if (((differ >> shift) & 2047) == 0) continue;
    uint32_t count[2049] = {0};
    for (size_t i = 0; i < n; ++i) count[((key[idx[i]] >> shift) & 2047) + 1]++;
    for (unsigned d = 0; d < 2048; ++d) count[d + 1] += count[d];
    for (size_t i = 0; i < n; ++i) tmp[count[(key[idx[i]] >> shift) & 2047]++] = idx[i];
    idx.swap(tmp);
  }
}

std::vector<uint32_t> identity(size_t n) {
  std::vector<uint32_t> v(n);
  std::iota(v.begin(), v.end(), 0u);
  return v;
}

}  // namespace

int ss_apply_core(const ss_config_t &cfg, const ss_policy_item_t *policy, uint32_t k, const int32_t *new_idx,
                  const ss_tensor_t *tensors, uint32_t n_tensors, ss_applied &out) {
  const uint64_t bpo = cfg.link_bytes_per_op;
  const uint64_t align = cfg.align, guard = cfg.guard_bytes;
  // (producer operator, output slot) -> row of the tensor table
  std::vector<uint64_t> row_key(n_tensors);
  std::vector<uint32_t> scratch;
  uint32_t max_op = 0;
  for (uint32_t r = 0; r < n_tensors; ++r) {
    row_key[r] = ((uint64_t)tensors[r].producer_op << 32) | tensors[r].out_slot;
    if (tensors[r].first_bwd_use != SS_NONE_OP) max_op = std::max(max_op, tensors[r].first_bwd_use);
  }
  const uint64_t bpo_in = cfg.prefetch_bytes_per_op ? cfg.prefetch_bytes_per_op : bpo;
  // link times are kept below 2^63
  if ((u128)(max_op + 2ull) * bpo >= ((u128)1 << 62)) return SS_E_INVAL;
  if ((u128)(max_op + 2ull) * bpo_in >= ((u128)1 << 62)) return SS_E_INVAL;
  std::vector<uint32_t> rows_sorted = identity(n_tensors);     // by (key, row)
  stable_sort_by(rows_sorted, row_key, scratch);
  std::vector<uint64_t> keys_sorted(n_tensors);
  for (uint32_t i = 0; i < n_tensors; ++i) keys_sorted[i] = row_key[rows_sorted[i]];
  auto find_row = [&](uint32_t op, uint32_t slot, uint32_t &row) {
    const uint64_t key = ((uint64_t)op << 32) | slot;
    auto it = std::lower_bound(keys_sorted.begin(), keys_sorted.end(), key);
    if (it == keys_sorted.end() || *it != key) return false;
    row = rows_sorted[it - keys_sorted.begin()];
    return true;
  };

  out = ss_applied();
  out.resolved.assign(policy, policy + k);
  std::vector<uint32_t> flags(k, 0);
  std::vector<Live> live;
  live.reserve(k);
  std::vector<uint8_t> claimed(n_tensors, 0);
  for (uint32_t a = 0; a < k; ++a) {
    uint32_t row;
    if (new_idx[a] < 0 || !find_row((uint32_t)new_idx[a], policy[a].out_slot, row)) {
      flags[a] |= SS_F_UNMATCHED;
      continue;
    }
    const ss_tensor_t &t = tensors[row];
    if (t.last_fwd_use == SS_NONE_OP || t.first_bwd_use == SS_NONE_OP || !(t.last_fwd_use < t.first_bwd_use)) {
      flags[a] |= SS_F_ORDER;
      continue;
    }
    if (claimed[row]) {               // a tensor is claimed once: the lower policy index keeps it
      flags[a] |= SS_F_UNMATCHED;
      continue;
    }
    claimed[row] = 1;
    Live L;
    L.a = a; L.row = row; L.t_out = t.last_fwd_use; L.t_use = t.first_bwd_use; L.nbytes = t.nbytes;
    live.push_back(L);
  }

  // live is in policy-index order, so a stable ordering by an operator index alone is "(operator, policy index)"
  std::vector<uint64_t> k_out(live.size()), k_use(live.size());
  for (size_t i = 0; i < live.size(); ++i) {
    k_out[i] = live[i].t_out;
    k_use[i] = live[i].t_use;
  }

  if (cfg.flags & SS_CFG_POLICY_POINTS) {
    // The generator already fixed release and pre-trigger points (Sec. 4.3, 4.4): keep them, moved
    // along with the tensor's own last forward use / first backward use in this iteration.
    for (Live &L : live) {
      const ss_policy_item_t &p = policy[L.a];
      int64_t tf = (int64_t)p.t_free + (int64_t)L.t_out - (int64_t)p.t_out;
      int64_t ti = (int64_t)p.t_in + (int64_t)L.t_use - (int64_t)p.t_use;
      bool ok = (int64_t)L.t_out <= tf && tf < ti && ti <= (int64_t)L.t_use;
      if (!ok && (cfg.flags & SS_CFG_KEEP_LATE)) {
        tf = std::min(std::max(tf, (int64_t)L.t_out), (int64_t)L.t_use - 1);
        ti = std::min(std::max(ti, tf + 1), (int64_t)L.t_use);
        ok = true;
        L.forced = true;
      }
      L.valid = ok;
      L.t_free = ok ? (uint64_t)tf : 0;
      L.t_in = ok ? (uint64_t)ti : 0;
      L.late = (p.flags & SS_F_LATE) != 0 || L.forced;
    }
    std::vector<uint32_t> need = identity(live.size());
    stable_sort_by(need, k_use, scratch);            // (t_use, policy index)
    uint64_t run = 0;                              // first-in first-out order of need
    for (uint32_t i : need) {
      Live &L = live[i];
      if (!L.valid) continue;
      L.t_in = std::max(L.t_in, run);
      run = L.t_in;
    }
  } else {
    // swap-out queue: FIFO in (t_out, policy index) order
    std::vector<uint32_t> ord = identity(live.size());
    stable_sort_by(ord, k_out, scratch);             // (t_out, policy index)
    uint64_t link_free = 0;
    for (uint32_t i : ord) {
      Live &L = live[i];
      const uint64_t ready = (L.t_out + 1) * bpo;
      const uint64_t start = std::max(ready, link_free);
      const uint64_t end = start + L.nbytes;
      if (end >= (1ull << 62)) return SS_E_INVAL;
      link_free = end;
      L.t_free = (end - 1) / bpo;          // the operator running when the last byte lands
      if (!(L.t_free < L.t_use)) {
        if (cfg.flags & SS_CFG_KEEP_LATE) {      // must be executed anyway: released and re-fetched around its use
          L.t_free = L.t_use - 1;
          L.forced = true;
        } else {
          L.valid = false;                       // saves no memory: dropped
        }
      }
    }
    // swap-in queue: as late as possible, walking (t_use, policy index) downwards
    ord = identity(live.size());
    stable_sort_by(ord, k_use, scratch);             // (t_use, policy index) upwards ...
    std::reverse(ord.begin(), ord.end());            // ... walked downwards
    // No swap-in is issued before the last swap-out has been issued: until then memory is still
    // climbing to its peak and a swap-in would only fight the swap-outs for the link (Sec. 4.3.1:
    // the search for a swap-in slot does not go back beyond the peak-memory period).
    uint64_t t_peak = 0;
    for (const Live &L : live)
      if (L.valid) t_peak = std::max(t_peak, L.t_out + 1);
    bool have_next = false;
    int64_t next_start = 0;
    for (uint32_t i : ord) {
      Live &L = live[i];
      if (!L.valid) continue;
      int64_t end = (int64_t)(L.t_use * bpo_in);
      if (have_next && next_start < end) end = next_start;
      int64_t start = end - (int64_t)L.nbytes;
      const int64_t floor_ = (int64_t)(std::max(L.t_free + 1, t_peak) * bpo_in);
      if (start < floor_) {
        start = floor_;
        L.late = true;
      }
      L.t_in = (uint64_t)start / bpo_in;
      next_start = start;
      have_next = true;
    }
    // The swap-in stream is first-in first-out: an item needed later is never issued before one
    // needed earlier (the release-point floor can otherwise put it ahead in the queue).
    {
      uint64_t run = 0;
      for (auto it = ord.rbegin(); it != ord.rend(); ++it) {     // (t_use, policy index) ascending
        Live &L = live[*it];
        if (!L.valid) continue;
        L.t_in = std::max(L.t_in, run);
        run = L.t_in;
      }
    }
  }

  // keep what satisfies t_out <= t_free < t_in <= t_use
  std::vector<uint32_t> kept;        // indices into live
  for (uint32_t i = 0; i < live.size(); ++i) {
    Live &L = live[i];
    if (!(L.valid && L.t_out <= L.t_free && L.t_free < L.t_in && L.t_in <= L.t_use)) {
      flags[L.a] |= SS_F_ORDER;
      continue;
    }
    if (L.late) flags[L.a] |= SS_F_LATE;
    if (L.forced) flags[L.a] |= SS_F_FORCED;
    if (L.nbytes != policy[L.a].nbytes) flags[L.a] |= SS_F_RESIZED;
    kept.push_back(i);
  }
  for (uint32_t a = 0; a < k; ++a) {
    ss_policy_item_t &r = out.resolved[a];
    r.flags = flags[a];
    r.t_out = r.t_free = r.t_in = r.t_use = 0;
  }
  for (uint32_t i : kept) {
    const Live &L = live[i];
    ss_policy_item_t &r = out.resolved[L.a];
    r.tensor_id = tensors[L.row].tensor_id;
    r.t_out = (uint32_t)L.t_out; r.t_free = (uint32_t)L.t_free;
    r.t_in = (uint32_t)L.t_in; r.t_use = (uint32_t)L.t_use;
    r.nbytes = L.nbytes;
    if (L.late) out.n_late++;
  }
  out.n_kept = (uint32_t)kept.size();
  out.n_dropped = k - out.n_kept;
  if (kept.empty()) {
    out.out_start.assign(1, 0);
    out.in_start.assign(1, 0);
    return SS_OK;
  }

  // queue ranks
  std::vector<uint32_t> out_order(kept), in_order(kept);
  stable_sort_by(out_order, k_out, scratch);         // kept is in policy-index order: (t_out, policy index)
  stable_sort_by(in_order, k_use, scratch);          // (t_use, policy index)

  // staging slots: exclusive prefix sum of aligned sizes (+ guard) in swap-out order
  std::vector<uint64_t> host_off(live.size(), 0);
  uint64_t off = guard;
  for (uint32_t i : out_order) {
    host_off[i] = off;
    off += ss_align_up(live[i].nbytes, align) + guard;
    out.bytes_out += live[i].nbytes;
  }
  out.staging_bytes = off;

  // swap-out batches: everything issued after the same operator
  std::vector<uint32_t> out_batch(live.size(), 0), in_batch(live.size(), 0);
  out.out_start.assign(1, 0);
  for (size_t p = 0; p < out_order.size(); ++p) {
    const uint32_t i = out_order[p];
    if (p && live[i].t_out != live[out_order[p - 1]].t_out) out.out_start.push_back((uint32_t)out.out.size());
    out_batch[i] = (uint32_t)out.out_start.size() - 1;
    const ss_tensor_t &t = tensors[live[i].row];
    out.out.push_back(ss_desc_t{t.dev_off, host_off[i], live[i].nbytes, t.tensor_id, flags[live[i].a]});
  }
  out.out_start.push_back((uint32_t)out.out.size());
  // swap-in batches: issued before the same operator and first used by the same operator, in swap-in queue order
  std::vector<uint32_t> in_issue(in_order);          // in swap-in rank order; now by (t_in, rank)
  {
    std::vector<uint64_t> k_in(live.size());
    for (size_t i = 0; i < live.size(); ++i) k_in[i] = live[i].t_in;
    stable_sort_by(in_issue, k_in, scratch);
  }
  out.in_start.assign(1, 0);
  for (size_t p = 0; p < in_issue.size(); ++p) {
    const uint32_t i = in_issue[p];
    // a batch: same issue point and same first use (so a wait covers only what that use needs)
    const bool fresh = p == 0 || live[i].t_in != live[in_issue[p - 1]].t_in ||
                       live[i].t_use != live[in_issue[p - 1]].t_use;
    if (p && fresh) out.in_start.push_back((uint32_t)out.in.size());
    if (fresh) out.in_dep.push_back(0);
    const uint32_t b = (uint32_t)out.in_start.size() - 1;
    in_batch[i] = b;
    out.in_dep[b] = std::max(out.in_dep[b], out_batch[i]);
    const ss_tensor_t &t = tensors[live[i].row];
    out.in.push_back(ss_desc_t{t.dev_off_in, host_off[i], live[i].nbytes, t.tensor_id, flags[live[i].a]});
  }
  out.in_start.push_back((uint32_t)out.in.size());

  // actions, sorted by (operator, kind, queue rank): listed kind after kind (IN < WAIT_IN < OUT < FREE)
  // in rank order, then ordered by operator alone with a stable pass
  {
    const size_t nk = kept.size();
    std::vector<ss_action_t> list;
    list.reserve(4 * nk);
    std::vector<uint64_t> op_of;
    op_of.reserve(4 * nk);
    auto push = [&](uint64_t op, uint32_t kind, uint32_t i, uint32_t batch) {
      list.push_back(ss_action_t{(uint32_t)op, kind, tensors[live[i].row].tensor_id, batch});
      op_of.push_back(op);
    };
    static_assert(SS_ACT_IN < SS_ACT_WAIT_IN && SS_ACT_WAIT_IN < SS_ACT_OUT && SS_ACT_OUT < SS_ACT_FREE, "kind order");
    for (uint32_t i : in_order) push(live[i].t_in, SS_ACT_IN, i, in_batch[i]);
    for (uint32_t i : in_order) push(live[i].t_use, SS_ACT_WAIT_IN, i, in_batch[i]);
    for (uint32_t i : out_order) push(live[i].t_out, SS_ACT_OUT, i, out_batch[i]);
    for (uint32_t i : out_order) push(live[i].t_free, SS_ACT_FREE, i, out_batch[i]);
    std::vector<uint32_t> order = identity(list.size());
    stable_sort_by(order, op_of, scratch);
    out.actions.reserve(list.size());
    for (uint32_t j : order) out.actions.push_back(list[j]);
  }

  // policy events for the timeline scan: release at t_free, allocation at t_in; operator
  // order, allocations first inside an operator, then swap-out rank
  {
    const size_t nk = kept.size();
    std::vector<ss_event_t> list;
    list.reserve(2 * nk);
    std::vector<uint64_t> op_of;
    op_of.reserve(2 * nk);
    for (uint32_t i : out_order) {
      list.push_back(ss_event_t{(uint32_t)live[i].t_in, tensors[live[i].row].tensor_id, (int64_t)live[i].nbytes});
      op_of.push_back(live[i].t_in);
    }
    for (uint32_t i : out_order) {
      list.push_back(ss_event_t{(uint32_t)live[i].t_free, tensors[live[i].row].tensor_id, -(int64_t)live[i].nbytes});
      op_of.push_back(live[i].t_free);
    }
    std::vector<uint32_t> order = identity(list.size());
    stable_sort_by(order, op_of, scratch);
    out.pevents.reserve(list.size());
    for (uint32_t j : order) out.pevents.push_back(list[j]);
  }
  return SS_OK;
}

extern "C" int ss_apply_policy(ss_ctx *ctx, const ss_policy_item_t *policy, uint32_t k, const int32_t *new_idx,
                               const ss_tensor_t *tensors, uint32_t n_tensors, ss_policy_item_t *resolved,
                               ss_action_t *actions, uint32_t *n_actions, ss_desc_t *descs_out,
                               ss_desc_t *descs_in, ss_event_t *pevents, uint32_t *n_pe,
                               ss_apply_result_t *res) {
  return ss_guard([&]() -> int {
    if (!ctx || !res || !n_actions || !n_pe) return SS_E_INVAL;
    if (k && (!policy || !new_idx || !actions || !descs_out || !descs_in || !pevents)) return SS_E_INVAL;
    if (n_tensors && !tensors) return SS_E_INVAL;
    ss_applied ap;
    int rc = ss_apply_core(ctx->cfg, policy, k, new_idx, tensors, n_tensors, ap);
    if (rc != SS_OK) return rc;
    if (ap.actions.size() > *n_actions || ap.pevents.size() > *n_pe) return SS_E_CAPACITY;
    if (resolved && k) std::memcpy(resolved, ap.resolved.data(), (size_t)k * sizeof(ss_policy_item_t));
    if (!ap.actions.empty()) std::memcpy(actions, ap.actions.data(), ap.actions.size() * sizeof(ss_action_t));
    if (!ap.out.empty()) std::memcpy(descs_out, ap.out.data(), ap.out.size() * sizeof(ss_desc_t));
    if (!ap.in.empty()) std::memcpy(descs_in, ap.in.data(), ap.in.size() * sizeof(ss_desc_t));
    if (!ap.pevents.empty()) std::memcpy(pevents, ap.pevents.data(), ap.pevents.size() * sizeof(ss_event_t));
    *n_actions = (uint32_t)ap.actions.size();
    *n_pe = (uint32_t)ap.pevents.size();
    std::memset(res, 0, sizeof(*res));
    res->staging_bytes = ap.staging_bytes;
    res->bytes_out = ap.bytes_out;
    res->n_kept = ap.n_kept;
    res->n_dropped = ap.n_dropped;
    res->n_late = ap.n_late;
    res->n_out_batches = (uint32_t)ap.out_start.size() - 1;
    res->n_in_batches = (uint32_t)ap.in_start.size() - 1;
    if (ap.staging_bytes > ctx->cfg.staging_bytes) return SS_E_NOMEM;
    if (!ctx->bound) return SS_OK;          // schedule computed; nothing to load it against yet
    rc = ss_load_schedule(ctx, ap.out.data(), (uint32_t)ap.out.size(), ap.out_start.data(), res->n_out_batches,
                          ap.in.data(), (uint32_t)ap.in.size(), ap.in_start.data(), res->n_in_batches,
                          ap.in_dep.data());
    if (rc != SS_OK) return rc;
    // keep the actions for ss_dispatch: they are sorted by (operator, kind), so the actions before an
    // operator (IN, WAIT_IN) and those after it (OUT, FREE) are two consecutive runs
    ss_sched &s = ctx->sched;
    s.actions = ap.actions;
    const uint64_t groups = s.actions.empty() ? 0 : 2ull * ((uint64_t)s.actions.back().op_idx + 1);
    s.act_start.assign(groups + 1, 0);
    for (const ss_action_t &a : s.actions) s.act_start[2ull * a.op_idx + (a.kind >= SS_ACT_OUT ? 1 : 0) + 1]++;
    for (uint64_t g = 0; g < groups; ++g) s.act_start[g + 1] += s.act_start[g];
    s.have_actions = true;
    // reuse interval of every kept item (Sec. 6.4): operators between issuing the swap-out and the release
    std::memset(ctx->stats.reuse_hist, 0, sizeof(ctx->stats.reuse_hist));
    ctx->stats.reuse_sum = ctx->stats.reuse_count = 0;
    for (const ss_policy_item_t &it : ap.resolved) {
      if (it.flags & (SS_F_UNMATCHED | SS_F_ORDER)) continue;
      const uint64_t gap = (uint64_t)it.t_free - it.t_out;
      uint32_t b = 0;
      while (b < 15 && ((gap + 1) >> (b + 1))) ++b;
      ctx->stats.reuse_hist[b]++;
      ctx->stats.reuse_sum += gap;
      ctx->stats.reuse_count++;
    }
    return SS_OK;
  });
}

extern "C" int ss_greedy_policy(ss_ctx *ctx, const ss_tensor_t *tensors, uint32_t n_tensors, const ss_event_t *ev,
                                uint64_t n_ev, uint32_t n_ops, int64_t base, int64_t budget, uint64_t min_bytes,
                                const ss_policy_item_t *initial, uint32_t n_initial,
                                ss_policy_item_t *policy_out, uint32_t *n_policy, int64_t *peak_out) {
  return ss_guard([&]() -> int {
    if (!ctx || !n_policy || (n_tensors && !tensors) || (n_initial && !initial)) return SS_E_INVAL;
    if (*n_policy && !policy_out) return SS_E_INVAL;
    const uint32_t cap = *n_policy;
    std::vector<ss_policy_item_t> rows(initial, initial + n_initial);
    std::vector<int32_t> idx;
    std::vector<int64_t> mre(n_ops);
    ss_scan_result_t sr;
    ss_applied ap;
    auto evaluate = [&](bool want_mre) -> int {
      idx.resize(rows.size());
      for (size_t i = 0; i < rows.size(); ++i) idx[i] = (int32_t)rows[i].ref_op;   // same iteration: identity
      int rc = ss_apply_core(ctx->cfg, rows.data(), (uint32_t)rows.size(), idx.data(), tensors, n_tensors, ap);
      if (rc != SS_OK) return rc;
      return ss_timeline_scan(ctx, ev, n_ev, ap.pevents.data(), ap.pevents.size(), n_ops, base, budget, nullptr,
                              nullptr, want_mre ? mre.data() : nullptr, &sr);
    };
    auto finish = [&]() -> int {
      if (rows.size() > cap) return SS_E_CAPACITY;
      if (!rows.empty()) std::memcpy(policy_out, rows.data(), rows.size() * sizeof(ss_policy_item_t));
      *n_policy = (uint32_t)rows.size();
      if (peak_out) *peak_out = sr.peak;
      return SS_OK;
    };
    int rc = evaluate(true);
    if (rc != SS_OK) return rc;
    if (sr.peak <= budget) return finish();

    // candidates: kept from forward to backward with room for a round trip, not too small, not
    // already chosen, idle span covering at least one over-budget operator (Sec. 4.2)
    std::vector<uint32_t> over_prefix(n_ops + 1, 0);        // over_prefix[t] = #over-budget operators < t
    for (uint32_t t = 0; t < n_ops; ++t) over_prefix[t + 1] = over_prefix[t] + (mre[t] > 0);
    std::vector<uint8_t> chosen(n_tensors, 0);
    {
      std::vector<std::pair<uint32_t, uint32_t>> by_id(n_tensors);
      for (uint32_t r = 0; r < n_tensors; ++r) by_id[r] = {tensors[r].tensor_id, r};
      std::sort(by_id.begin(), by_id.end());
      for (const ss_policy_item_t &p : rows) {
        auto it = std::lower_bound(by_id.begin(), by_id.end(), std::make_pair(p.tensor_id, 0u));
        if (it != by_id.end() && it->first == p.tensor_id) chosen[it->second] = 1;
      }
    }
    std::vector<uint32_t> cand;
    for (uint32_t r = 0; r < n_tensors; ++r) {
      const ss_tensor_t &t = tensors[r];
      if (t.last_fwd_use == SS_NONE_OP || t.first_bwd_use == SS_NONE_OP) continue;
      if (!((uint64_t)t.last_fwd_use + 1 < t.first_bwd_use) || t.first_bwd_use > n_ops) continue;
      if (t.nbytes < min_bytes || chosen[r]) continue;
      if (over_prefix[t.first_bwd_use] - over_prefix[t.last_fwd_use + 1] == 0) continue;
      cand.push_back(r);
    }
    std::sort(cand.begin(), cand.end(), [&](uint32_t x, uint32_t y) {
      const ss_tensor_t &a = tensors[x], &b = tensors[y];
      const uint32_t ia = a.first_bwd_use - a.last_fwd_use, ib = b.first_bwd_use - b.last_fwd_use;
      if (ia != ib) return ia > ib;                          // longest idle span first
      if (a.nbytes != b.nbytes) return a.nbytes > b.nbytes;  // then larger first
      return a.tensor_id < b.tensor_id;
  });
  for (uint32_t r : cand) {
    const ss_tensor_t &t = tensors[r];
    ss_policy_item_t p;
    std::memset(&p, 0, sizeof(p));
    p.ref_op = t.producer_op; p.out_slot = t.out_slot; p.tensor_id = t.tensor_id; p.nbytes = t.nbytes;
    rows.push_back(p);
    if ((rc = evaluate(false)) != SS_OK) return rc;
    if (sr.peak <= budget) return finish();
  }
  if (peak_out) *peak_out = sr.peak;
  return SS_E_INFEASIBLE;
  });
}
