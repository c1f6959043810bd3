// Policy generator (Sec. 4 of the SmartSwap paper): logical layers with the time estimate of
// Eq. 1, the memory reduction list, the candidate list ranked by Eq. 2, the swap simulator
// (pre-triggered swap-in, Eq. 3; swap-out completion) and the loop of Algo. 2.  The memory curve
// without swaps and the check of the finished policy are timeline scans on the GPU; the
// simulator itself is sequential integer work on the host.  Time is counted in link bytes, so a
// transfer costs its size and a layer owns link_bytes_per_op times its operator count.
#include <algorithm>
#include <cstring>

#include "ss_internal.h"

namespace {

struct Layer {
  uint32_t first, end;     // operators [first, end)
  uint32_t type;           // 0 forward, 1 backward, 2 optimizer
  int64_t remaining;       // link bytes still free in this layer
  uint64_t bpo;            // link bytes one operator of this layer is worth (Eq. 1)
};

struct Chosen {
  uint32_t row, layer_in, t_in, t_free;
  bool late;
};

typedef unsigned __int128 u128;

// Cut the operators of each phase, in execution order, into groups of (almost) equal count.
void build_layers(const std::vector<uint32_t> &phase, uint32_t g_fwd, uint32_t g_bwd, const uint64_t bpo[3],
                  std::vector<Layer> &layers, std::vector<uint32_t> &layer_of) {
  const uint32_t n = (uint32_t)phase.size();
  struct Raw { Layer L; std::vector<uint32_t> ops; };
  std::vector<Raw> raw;
  const uint32_t groups[3] = {g_fwd, g_bwd, 1};
  for (uint32_t ph = 0; ph < 3; ++ph) {
    std::vector<uint32_t> idx;
    for (uint32_t i = 0; i < n; ++i)
      if (phase[i] == ph) idx.push_back(i);
    if (idx.empty()) continue;
    const uint64_t G = std::max<uint64_t>(1, std::min<uint64_t>(groups[ph], idx.size()));
    for (uint64_t g = 0; g < G; ++g) {
      const size_t lo = (size_t)(g * idx.size() / G), hi = (size_t)((g + 1) * idx.size() / G);
      if (hi <= lo) continue;
      Raw r;
      r.L = Layer{idx[lo], idx[hi - 1] + 1, ph, (int64_t)(bpo[ph] * (hi - lo)), bpo[ph]};
      r.ops.assign(idx.begin() + lo, idx.begin() + hi);
      raw.push_back(std::move(r));
    }
  }
  std::sort(raw.begin(), raw.end(), [](const Raw &a, const Raw &b) { return a.L.first < b.L.first; });
  layers.clear();
  layer_of.assign(n, 0);
  for (size_t li = 0; li < raw.size(); ++li) {
    layers.push_back(raw[li].L);
    for (uint32_t i : raw[li].ops) layer_of[i] = (uint32_t)li;
  }
}

}  // namespace

// The generator proper: per_op is the memory without swaps (n_ops entries).  Fills `items` in commit
// order and the counters of `res` that do not need a scan.
static int generate_core(uint64_t bpo, const ss_op_t *ops, uint32_t n_ops, const ss_tensor_t *tensors,
                         uint32_t n_tensors, const std::vector<int64_t> &per_op, int64_t limit,
                         const ss_gen_params_t *params, std::vector<ss_policy_item_t> &items,
                         std::vector<ss_event_t> &pe, ss_gen_result_t *res) {
  if (params->c_den == 0 || params->g_fwd == 0 || params->g_bwd == 0) return SS_E_INVAL;
  std::vector<int64_t> excess(n_ops, 0);
  uint32_t n_entries = 0;
  for (uint32_t t = 0; t < n_ops; ++t)
    if (per_op[t] > limit) { excess[t] = per_op[t] - limit; ++n_entries; }
  std::vector<uint32_t> phase(n_ops);
  for (uint32_t i = 0; i < n_ops; ++i) phase[i] = std::min<uint32_t>(ops[i].sig >> 16, 2u);
  std::vector<Layer> layers;
  std::vector<uint32_t> layer_of;
  uint64_t bpo3[3];
  for (int ph = 0; ph < 3; ++ph) bpo3[ph] = params->phase_bytes_per_op[ph] ? params->phase_bytes_per_op[ph] : bpo;
  build_layers(phase, params->g_fwd, params->g_bwd, bpo3, layers, layer_of);

  // entries the tensor can be away from: operators t with last_fwd_use + 1 < t < first_bwd_use
  auto span_count = [&](const ss_tensor_t &t, int64_t &last) {
    uint32_t c = 0;
    last = -1;
    for (uint64_t op = (uint64_t)t.last_fwd_use + 2; op < t.first_bwd_use && op < n_ops; ++op)
      if (excess[op] > 0) { ++c; last = (int64_t)op; }
    return c;
  };
  auto usable = [&](const ss_tensor_t &t) {
    return t.last_fwd_use != SS_NONE_OP && t.first_bwd_use != SS_NONE_OP && t.last_fwd_use < t.first_bwd_use &&
           t.first_bwd_use < n_ops && t.nbytes >= params->min_bytes;
  };

  std::vector<uint8_t> taken(n_tensors, 0);
  std::vector<Chosen> chosen;
  auto commit = [&](uint32_t row, uint32_t L_in, bool late) {
    const ss_tensor_t &t = tensors[row];
    const uint32_t t_in = layers[L_in].first;
    layers[L_in].remaining -= (int64_t)t.nbytes;
    for (uint64_t op = (uint64_t)t.last_fwd_use + 2; op < t_in; ++op)
      if (excess[op] > 0) {
        excess[op] -= (int64_t)t.nbytes;
        if (excess[op] <= 0) { excess[op] = 0; --n_entries; }
      }
    taken[row] = 1;
    chosen.push_back(Chosen{row, L_in, t_in, 0, late});
  };

  struct Cand { uint32_t row, n_mre; uint64_t size; u128 key; };
  while (n_entries) {                                   // Algo. 2
    std::vector<Cand> cl;
    uint32_t max_n = 0;
    uint64_t max_s = 0;
    for (uint32_t r = 0; r < n_tensors; ++r) {
      if (taken[r] || !usable(tensors[r])) continue;
      int64_t last;
      const uint32_t c = span_count(tensors[r], last);
      if (!c) continue;
      cl.push_back(Cand{r, c, tensors[r].nbytes, 0});
      max_n = std::max(max_n, c);
      max_s = std::max(max_s, tensors[r].nbytes);
    }
    if (cl.empty()) return SS_E_INFEASIBLE;             // "Raise Error"
    for (Cand &c : cl)                                  // Eq. 2, scaled to integers
      c.key = (u128)c.n_mre * max_s * params->c_den + (u128)params->c_num * c.size * max_n;
    std::sort(cl.begin(), cl.end(), [&](const Cand &a, const Cand &b) {
      if (a.key != b.key) return a.key > b.key;
      if (a.size != b.size) return a.size > b.size;
      return tensors[a.row].tensor_id < tensors[b.row].tensor_id;
    });
    res->n_rounds++;

    uint32_t committed = 0;
    for (const Cand &c : cl) {                          // pre-trigger swap-in (Sec. 4.3.1)
      if (!n_entries) break;
      const ss_tensor_t &t = tensors[c.row];
      int64_t last;
      if (!span_count(t, last)) continue;
      const uint32_t L_use = layer_of[t.first_bwd_use], L_peak = layer_of[(uint32_t)last];
      for (int64_t L = (int64_t)L_use - 1; L > (int64_t)L_peak; --L)
        if (layers[(size_t)L].remaining > (int64_t)t.nbytes) {
          commit(c.row, (uint32_t)L, false);
          ++committed;
          break;
        }
    }
    if (!committed && n_entries) {                      // accept latency rather than stop
      for (const Cand &c : cl) {
        const ss_tensor_t &t = tensors[c.row];
        int64_t last;
        if (!span_count(t, last)) continue;
        const uint32_t L_use = layer_of[t.first_bwd_use];
        const uint32_t L_in = std::max<uint32_t>(L_use ? L_use - 1 : 0, layer_of[t.last_fwd_use] + 1);
        if (L_in > L_use) continue;
        commit(c.row, L_in, true);
        ++committed;
        break;
      }
      if (!committed) return SS_E_INFEASIBLE;
    }
  }

  // SetFreeTime: swap-out completion in swap-out order (Sec. 4.3.2)
  std::vector<uint32_t> order(chosen.size());
  for (uint32_t i = 0; i < order.size(); ++i) order[i] = i;
  std::sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) {
    const ss_tensor_t &a = tensors[chosen[x].row], &b = tensors[chosen[y].row];
    return a.last_fwd_use != b.last_fwd_use ? a.last_fwd_use < b.last_fwd_use : a.tensor_id < b.tensor_id;
  });
  for (uint32_t i : order) {
    Chosen &c = chosen[i];
    const ss_tensor_t &t = tensors[c.row];
    const uint32_t L0 = layer_of[t.last_fwd_use];
    const int64_t last = (int64_t)c.layer_in - 1;
    int64_t found = -1;
    for (int64_t L = L0; L <= last; ++L) {
      int64_t avail = layers[(size_t)L].remaining;
      if (L == (int64_t)L0) {
        // the swap-out starts right after the last forward use: of that use's own layer only the operators
        // that follow it can carry the transfer
        uint64_t after = 0;
        for (uint64_t op = (uint64_t)t.last_fwd_use + 1; op < layers[(size_t)L].end; ++op)
          after += layer_of[op] == (uint32_t)L;
        avail = std::min<int64_t>(avail, (int64_t)(layers[(size_t)L].bpo * after));
      }
      if (avail > (int64_t)t.nbytes) { found = L; break; }
    }
    if (found < 0) {
      found = std::max<int64_t>(L0, last);
      c.late = true;
    }
    layers[(size_t)found].remaining -= (int64_t)t.nbytes;
    const uint32_t end_op = layers[(size_t)found].end - 1;
    c.t_free = std::min<uint32_t>(std::max<uint32_t>(end_op, t.last_fwd_use + 1), c.t_in - 1);
  }

  items.clear();
  pe.clear();
  pe.reserve(2 * chosen.size());
  for (size_t i = 0; i < chosen.size(); ++i) {
    const Chosen &c = chosen[i];
    const ss_tensor_t &t = tensors[c.row];
    ss_policy_item_t p;
    std::memset(&p, 0, sizeof(p));
    p.ref_op = t.producer_op; p.out_slot = t.out_slot; p.tensor_id = t.tensor_id;
    p.flags = c.late ? SS_F_LATE : 0;
    p.t_out = t.last_fwd_use; p.t_free = c.t_free; p.t_in = c.t_in; p.t_use = t.first_bwd_use;
    p.nbytes = t.nbytes;
    items.push_back(p);
    res->bytes += t.nbytes;
    res->n_late += c.late;
    pe.push_back(ss_event_t{c.t_free, t.tensor_id, -(int64_t)t.nbytes});
    pe.push_back(ss_event_t{c.t_in, t.tensor_id, (int64_t)t.nbytes});
  }
  res->n_items = (uint32_t)chosen.size();
  std::stable_sort(pe.begin(), pe.end(), [](const ss_event_t &a, const ss_event_t &b) { return a.op_idx < b.op_idx; });
  return SS_OK;
}

extern "C" int ss_generate_policy(ss_ctx *ctx, const ss_op_t *ops, uint32_t n_ops, const ss_tensor_t *tensors,
                                  uint32_t n_tensors, const ss_event_t *ev, uint64_t n_ev, int64_t base,
                                  int64_t limit, const ss_gen_params_t *params, ss_policy_item_t *policy_out,
                                  uint32_t *n_policy, ss_gen_result_t *res) {
  return ss_guard([&]() -> int {
    uint32_t chosen = 0;
    return ss_generate_policy_best(ctx, ops, n_ops, tensors, n_tensors, ev, n_ev, base, limit, params, 1, policy_out,
                                   n_policy, &chosen, res);
  });
}

extern "C" int ss_generate_policy_best(ss_ctx *ctx, const ss_op_t *ops, uint32_t n_ops, const ss_tensor_t *tensors,
                                       uint32_t n_tensors, const ss_event_t *ev, uint64_t n_ev, int64_t base,
                                       int64_t limit, const ss_gen_params_t *params, uint32_t n_params,
                                       ss_policy_item_t *policy_out, uint32_t *n_policy, uint32_t *chosen,
                                       ss_gen_result_t *res) {
  return ss_guard([&]() -> int {
    if (!ctx || !params || !n_params || !n_policy || !chosen || !res || (n_ops && !ops) || (n_tensors && !tensors))
      return SS_E_INVAL;
    if (*n_policy && !policy_out) return SS_E_INVAL;
    const uint64_t bpo = ctx->cfg.link_bytes_per_op;
    if ((u128)bpo * (n_ops + 1ull) >= ((u128)1 << 62)) return SS_E_INVAL;
    for (uint32_t c = 0; c < n_params; ++c) {
      if (params[c].c_den == 0 || params[c].g_fwd == 0 || params[c].g_bwd == 0) return SS_E_INVAL;
      for (int ph = 0; ph < 3; ++ph)
        if ((u128)params[c].phase_bytes_per_op[ph] * (n_ops + 1ull) >= ((u128)1 << 62)) return SS_E_INVAL;
    }
    std::memset(res, 0, sizeof(*res));

    // memory without swaps -> memory reduction list (Sec. 4.2)
    std::vector<int64_t> per_op(n_ops);
    ss_scan_result_t sr;
    int rc = ss_timeline_scan(ctx, ev, n_ev, nullptr, 0, n_ops, base, limit, nullptr, per_op.data(), nullptr, &sr);
    if (rc != SS_OK) return rc;
    const int64_t peak_no_swap = sr.peak;

    struct Cand { std::vector<ss_policy_item_t> items; std::vector<ss_event_t> pe; ss_gen_result_t r; int rc; };
    std::vector<Cand> cands(n_params);
    std::vector<ss_event_t> all_pe;
    std::vector<uint64_t> pe_start(n_params + 1, 0);
    bool any = false;
    for (uint32_t c = 0; c < n_params; ++c) {
      std::memset(&cands[c].r, 0, sizeof(ss_gen_result_t));
      cands[c].rc = generate_core(bpo, ops, n_ops, tensors, n_tensors, per_op, limit, &params[c], cands[c].items,
                                  cands[c].pe, &cands[c].r);
      if (cands[c].rc != SS_OK && cands[c].rc != SS_E_INFEASIBLE) return cands[c].rc;
      if (cands[c].rc != SS_OK) cands[c].pe.clear();
      any = any || cands[c].rc == SS_OK;
      all_pe.insert(all_pe.end(), cands[c].pe.begin(), cands[c].pe.end());
      pe_start[c + 1] = all_pe.size();
    }
    if (!any) return SS_E_INFEASIBLE;
    // what the release points really give: every candidate scanned with its own events, one launch
    std::vector<ss_scan_result_t> scans(n_params);
    rc = ss_timeline_scan_batch(ctx, ev, n_ev, all_pe.data(), pe_start.data(), n_params, n_ops, base, limit, nullptr,
                                scans.data());
    if (rc != SS_OK) return rc;
    int best = -1;
    for (uint32_t c = 0; c < n_params; ++c) {
      if (cands[c].rc != SS_OK) continue;
      cands[c].r.peak_no_swap = peak_no_swap;
      cands[c].r.peak_with_policy = scans[c].peak;
      cands[c].r.n_over_with_policy = scans[c].n_over;
      if (best < 0) { best = (int)c; continue; }
      const ss_gen_result_t &x = cands[c].r, &y = cands[best].r;
      // within the limit first, then fewer items that cost latency, then fewer bytes over the link
      const bool xf = x.n_over_with_policy == 0, yf = y.n_over_with_policy == 0;
      if (xf != yf) { if (xf) best = (int)c; continue; }
      if (!xf && x.n_over_with_policy != y.n_over_with_policy) {
        if (x.n_over_with_policy < y.n_over_with_policy) best = (int)c;
        continue;
      }
      if (x.n_late != y.n_late) { if (x.n_late < y.n_late) best = (int)c; continue; }
      if (x.bytes < y.bytes) best = (int)c;
    }
    const Cand &w = cands[(size_t)best];
    if (w.items.size() > *n_policy) return SS_E_CAPACITY;
    if (!w.items.empty()) std::memcpy(policy_out, w.items.data(), w.items.size() * sizeof(ss_policy_item_t));
    *n_policy = (uint32_t)w.items.size();
    *chosen = (uint32_t)best;
    *res = w.r;
    return SS_OK;
  });
}
