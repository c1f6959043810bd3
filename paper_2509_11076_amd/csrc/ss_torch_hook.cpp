// Online profiler hook inside PyTorch (Sec. 3 of the SmartSwap paper): a callback at the operator
// dispatch point that feeds ss_trace_record, in the two modes the paper describes.
//   Lightweight: one integer record per dispatched operator (its token and the phase), nothing else.
//   Detailed:    also a hash of the Python call stack, the data type and output count of the operator
//                (known when it returns) and the caching allocator's alloc / free calls as events.
// The dispatch point is ATen's RecordFunction (scope FUNCTION: every operator, also those an autograd
// node runs during backward); the allocator's calls come from its trace tracker.  Plain C ABI, loaded
// with ctypes beside libss.so; no Python module, no torch types in the signatures.
#include <Python.h>
#include <frameobject.h>
#include <ATen/record_function.h>
#include <c10/hip/HIPCachingAllocator.h>

#include <atomic>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "ss.h"
#include "ss_torch_hook.h"

namespace {

struct Hook {
  std::mutex mu;
  ss_ctx *ctx = nullptr;
  std::atomic<int> mode{SS_HOOK_OFF};
  std::atomic<uint32_t> phase{0};             // set by the training loop: 0 forward, 1 backward, 2 optimizer
  std::atomic<int> paused{0};                 // > 0: operators dispatched now are the executor's own, not the model's
  bool have_cb = false, have_tracker = false;
  at::CallbackHandle handle = 0;
  // operator name -> interned record, keyed by a 64-bit hash of the characters and verified by
  // comparison (a name's address is not an identity: some names are temporaries)
  struct Named { std::string name; ss_op_t op; };
  std::unordered_multimap<uint64_t, Named> by_name;
  std::unordered_map<uint64_t, uint32_t> live;        // allocator address -> event tensor id
  uint32_t next_id = 0;
  // Detailed mode's tensor table: one row per block allocated in this iteration, its uses filled in
  // from the operators' input lists
  std::vector<ss_tensor_t> table;
  std::map<uint64_t, uint32_t> by_addr;               // start address of a live block -> row
  uint32_t slot_op = SS_NONE_OP, slot_next = 0;       // output slots count up within one operator
  ss_hook_stats_t st{};
};
Hook g;

struct OpCtx : at::ObserverContext {
  uint32_t op_idx = 0;
  bool recorded = false;
};

uint32_t fnv1a32(const void *data, size_t n, uint32_t h = 2166136261u) {
  const uint8_t *p = (const uint8_t *)data;
  for (size_t i = 0; i < n; ++i) h = (h ^ p[i]) * 16777619u;
  return h;
}

// hash of (code object, line) of the innermost Python frames; 0 on a thread the interpreter does
// not know (operators that an autograd node runs on the engine's own thread).  PyTorch releases the
// interpreter lock before it dispatches an operator, so it is taken here for the walk; the caller
// holds none of this library's locks meanwhile (the allocator may call back with that lock held).
uint32_t python_stack_hash() {
  if (!Py_IsInitialized() || !PyGILState_GetThisThreadState()) return 0;
  struct Gil {
    PyGILState_STATE s = PyGILState_Ensure();
    ~Gil() { PyGILState_Release(s); }
  } gil;
  PyFrameObject *f = PyEval_GetFrame();           // borrowed
  if (!f) return 0;
  Py_INCREF(f);
  uint32_t h = 2166136261u;
  for (int depth = 0; f && depth < 8; ++depth) {
    PyCodeObject *code = PyFrame_GetCode(f);      // new reference
    const uint64_t rec[2] = {(uint64_t)(uintptr_t)code, (uint64_t)PyFrame_GetLineNumber(f)};
    h = fnv1a32(rec, sizeof(rec), h);
    Py_XDECREF(code);
    PyFrameObject *back = PyFrame_GetBack(f);     // new reference or NULL
    Py_DECREF(f);
    f = back;
  }
  Py_XDECREF(f);
  return h ? h : 1u;
}

uint32_t dtype_code(const at::Tensor &t) {
  switch (t.scalar_type()) {
    case at::kBFloat16: return 1;
    case at::kFloat: return 2;
    case at::kByte: return 3;
    case at::kHalf: return 4;
    case at::kLong: return 5;
    case at::kInt: return 6;
    case at::kBool: return 7;
    case at::kDouble: return 8;
    default: return 15;
  }
}

std::unique_ptr<at::ObserverContext> on_start(const at::RecordFunction &fn) {
  const int mode = g.mode.load(std::memory_order_relaxed);
  if (mode == SS_HOOK_OFF || g.paused.load(std::memory_order_relaxed) > 0) return nullptr;
  const uint32_t stack_hash = mode == SS_HOOK_DETAILED ? python_stack_hash() : 0u;
  std::lock_guard<std::mutex> lock(g.mu);
  if (!g.ctx) return nullptr;
  const char *name = fn.name();
  uint64_t hname = 1469598103934665603ull;
  for (const char *p = name; *p; ++p) hname = (hname ^ (uint8_t)*p) * 1099511628211ull;
  auto range = g.by_name.equal_range(hname);
  auto it = range.first;
  while (it != range.second && std::strcmp(it->second.name.c_str(), name) != 0) ++it;
  if (it == range.second) {
    ss_op_t fresh;
    if (ss_intern_op(g.ctx, name, "", 0, 0, 0, &fresh) != SS_OK) {
      g.st.errors++;
      return nullptr;
    }
    it = g.by_name.emplace(hname, Hook::Named{name, fresh});
  }
  ss_op_t op = it->second.op;
  op.sig = g.phase.load(std::memory_order_relaxed) << 16;
  op.stack_hash = stack_hash;
  uint32_t idx = 0;
  const ss_op_t *ops = nullptr;
  ss_trace_view(g.ctx, &ops, &idx, nullptr, nullptr, nullptr);
  if (ss_trace_record(g.ctx, &op, nullptr, 0) != SS_OK) {
    g.st.dropped_ops++;
    return nullptr;
  }
  g.st.ops++;
  if (mode != SS_HOOK_DETAILED) return nullptr;
  {
    const uint32_t phase = op.sig >> 16;
    auto use = [&](const at::Tensor &t) {
      if (!t.defined() || !t.has_storage()) return;
      const uint64_t p = (uint64_t)(uintptr_t)t.storage().data();
      auto it2 = g.by_addr.upper_bound(p);
      if (it2 == g.by_addr.begin()) return;
      --it2;
      ss_tensor_t &row = g.table[it2->second];
      if (p >= it2->first + row.nbytes) return;          // a block from before the iteration
      if (phase == 0) {
        if (row.last_fwd_use != SS_NONE_OP && idx > row.last_fwd_use) row.last_fwd_use = idx;
      } else if (row.first_bwd_use == SS_NONE_OP) {
        row.first_bwd_use = idx;
      }
    };
    for (const c10::IValue &v : fn.inputs()) {
      if (v.isTensor()) use(v.toTensor());
      else if (v.isTensorList())
        for (const at::Tensor &t : v.toTensorVector()) use(t);
    }
  }
  auto c = std::make_unique<OpCtx>();
  c->op_idx = idx;
  c->recorded = true;
  return c;
}

void on_end(const at::RecordFunction &fn, at::ObserverContext *raw) {
  OpCtx *c = static_cast<OpCtx *>(raw);
  if (!c || !c->recorded) return;
  uint32_t n_out = 0, dtype = 0;
  for (const c10::IValue &v : fn.outputs()) {
    if (v.isTensor() && v.toTensor().defined()) {
      if (n_out == 0) dtype = dtype_code(v.toTensor());
      ++n_out;
    }
  }
  std::lock_guard<std::mutex> lock(g.mu);
  if (g.ctx && ss_trace_amend(g.ctx, c->op_idx, dtype, n_out) != SS_OK) g.st.errors++;
  for (const c10::IValue &v : fn.outputs()) {             // the blocks the outputs live in get their type
    if (!v.isTensor() || !v.toTensor().defined() || !v.toTensor().has_storage()) continue;
    auto it = g.by_addr.find((uint64_t)(uintptr_t)v.toTensor().storage().data());
    if (it != g.by_addr.end() && g.table[it->second].dtype == 0) g.table[it->second].dtype = dtype_code(v.toTensor());
  }
}

void on_allocator(const c10::hip::HIPCachingAllocator::TraceEntry &e) {
  using TE = c10::hip::HIPCachingAllocator::TraceEntry;
  if (g.mode.load(std::memory_order_relaxed) != SS_HOOK_DETAILED) return;
  if (e.action_ != TE::ALLOC && e.action_ != TE::FREE_COMPLETED) return;
  std::lock_guard<std::mutex> lock(g.mu);
  if (!g.ctx) return;
  int rc;
  uint32_t cur_op = 0;
  ss_trace_view(g.ctx, nullptr, &cur_op, nullptr, nullptr, nullptr);
  if (e.action_ == TE::ALLOC) {
    const uint32_t id = g.next_id++;
    g.live[(uint64_t)e.addr_] = id;
    rc = ss_trace_event(g.ctx, id, (int64_t)e.size_);
    if (rc == SS_OK) {                                    // cur_op >= 1: the running operator is cur_op - 1
      const uint32_t op = cur_op - 1;
      if (g.slot_op != op) { g.slot_op = op; g.slot_next = 0; }
      const ss_op_t *ops = nullptr;
      ss_trace_view(g.ctx, &ops, nullptr, nullptr, nullptr, nullptr);
      const bool fwd = (ops[op].sig >> 16) == 0;
      ss_tensor_t row{};
      // a block the executor itself asks for (a swapped tensor's new place) is nobody's output slot
      const bool own = g.paused.load(std::memory_order_relaxed) > 0;
      row.tensor_id = id; row.producer_op = op; row.out_slot = own ? SS_NONE_OP : g.slot_next++; row.alloc_op = op;
      row.last_fwd_use = fwd ? op : SS_NONE_OP; row.first_bwd_use = SS_NONE_OP; row.free_op = SS_NONE_OP;
      row.nbytes = (uint64_t)e.size_;
      g.by_addr[(uint64_t)e.addr_] = (uint32_t)g.table.size();
      g.table.push_back(row);
    }
  } else {
    auto bt = g.by_addr.find((uint64_t)e.addr_);
    if (bt != g.by_addr.end()) {
      if (cur_op) g.table[bt->second].free_op = cur_op - 1;
      g.by_addr.erase(bt);
    }
    auto it = g.live.find((uint64_t)e.addr_);
    if (it == g.live.end()) {          // allocated before this iteration's record began: an id of its own
      g.st.foreign_frees++;
      rc = ss_trace_event(g.ctx, g.next_id++, -(int64_t)e.size_);
    } else {
      rc = ss_trace_event(g.ctx, it->second, -(int64_t)e.size_);
      g.live.erase(it);
    }
  }
  if (rc == SS_OK) g.st.events++;
  else g.st.dropped_events++;
}

// the callback's needs are fixed when it is registered: Lightweight asks for nothing (no boxing of
// outputs, no end callback), Detailed for the outputs
void register_callback(int mode) {
  // the allocator offers no way to detach a tracker, and an attached one costs a little on every
  // allocation: it is attached when Detailed mode is first asked for and stays
  if (mode == SS_HOOK_DETAILED && !g.have_tracker) {
    c10::hip::HIPCachingAllocator::attachAllocatorTraceTracker(on_allocator);
    g.have_tracker = true;
  }
  if (g.have_cb) {
    at::removeCallback(g.handle);
    g.have_cb = false;
  }
  if (mode == SS_HOOK_OFF) return;
  auto cb = mode == SS_HOOK_DETAILED ? at::RecordFunctionCallback(on_start, on_end).needsInputs(true).needsOutputs(true)
                                     : at::RecordFunctionCallback(on_start, nullptr);
  g.handle = at::addGlobalCallback(cb.scopes({at::RecordScope::FUNCTION}));
  g.have_cb = true;
}

// PyTorch reports failures by C++ exceptions (c10::Error); none may cross the C boundary
template <class Body>
int guarded(Body &&body) noexcept {
  try {
    return body();
  } catch (const std::bad_alloc &) {
    return SS_E_NOMEM;
  } catch (...) {
    std::lock_guard<std::mutex> lock(g.mu);
    g.st.errors++;
    return SS_E_STATE;
  }
}

}  // namespace

extern "C" int ss_hook_install(ss_ctx *ctx, int mode) {
  if (!ctx || mode < SS_HOOK_OFF || mode > SS_HOOK_DETAILED) return SS_E_INVAL;
  return guarded([&]() -> int {
    {
      std::lock_guard<std::mutex> lock(g.mu);
      if (g.ctx != ctx) g.by_name.clear();       // tokens are per context
      g.ctx = ctx;
    }
    register_callback(mode);
    g.mode.store(mode);
    return SS_OK;
  });
}

extern "C" int ss_hook_set_mode(int mode) {
  if (mode < SS_HOOK_OFF || mode > SS_HOOK_DETAILED) return SS_E_INVAL;
  return guarded([&]() -> int {
    if (mode != g.mode.load()) register_callback(mode);
    g.mode.store(mode);
    return SS_OK;
  });
}

extern "C" int ss_hook_set_phase(uint32_t phase) {
  if (phase > 2) return SS_E_INVAL;
  g.phase.store(phase);
  return SS_OK;
}

extern "C" int ss_hook_begin_iteration(void) {
  std::lock_guard<std::mutex> lock(g.mu);
  if (!g.ctx) return SS_E_INVAL;
  g.live.clear();
  g.next_id = 0;
  g.table.clear();
  g.by_addr.clear();
  g.slot_op = SS_NONE_OP;
  g.phase.store(0);
  return ss_trace_begin(g.ctx);
}

extern "C" int ss_hook_remove(void) {
  return guarded([&]() -> int {
    g.mode.store(SS_HOOK_OFF);
    register_callback(SS_HOOK_OFF);
    std::lock_guard<std::mutex> lock(g.mu);
    g.ctx = nullptr;
    g.by_name.clear();
    g.live.clear();
    return SS_OK;
  });
}

extern "C" int ss_hook_tensor_table(ss_tensor_t *out, uint32_t *n) {
  if (!n || (*n && !out)) return SS_E_INVAL;
  std::lock_guard<std::mutex> lock(g.mu);
  if (!g.ctx) return SS_E_STATE;
  const uint32_t have = (uint32_t)g.table.size();
  if (*n < have) { *n = have; return SS_E_CAPACITY; }
  uint32_t n_ops = 0;
  ss_trace_view(g.ctx, nullptr, &n_ops, nullptr, nullptr, nullptr);
  for (uint32_t i = 0; i < have; ++i) {
    out[i] = g.table[i];
    if (out[i].free_op == SS_NONE_OP && n_ops) out[i].free_op = n_ops - 1;   // still held when the iteration ends
  }
  *n = have;
  return SS_OK;
}

extern "C" int ss_hook_pause(int on) {
  if (on) g.paused.fetch_add(1);
  else if (g.paused.load() > 0) g.paused.fetch_sub(1);
  else return SS_E_STATE;
  return SS_OK;
}

extern "C" int ss_hook_current_op(uint32_t *n_ops) {
  if (!n_ops) return SS_E_INVAL;
  std::lock_guard<std::mutex> lock(g.mu);
  if (!g.ctx) return SS_E_STATE;
  return ss_trace_view(g.ctx, nullptr, n_ops, nullptr, nullptr, nullptr);
}

extern "C" int ss_hook_block_of(const void *dev_addr, ss_tensor_t *row, uint64_t *block_addr) {
  if (!dev_addr || !row) return SS_E_INVAL;
  std::lock_guard<std::mutex> lock(g.mu);
  if (!g.ctx) return SS_E_STATE;
  const uint64_t p = (uint64_t)(uintptr_t)dev_addr;
  auto it = g.by_addr.upper_bound(p);
  if (it == g.by_addr.begin()) return SS_E_INVAL;
  --it;
  if (p >= it->first + g.table[it->second].nbytes) return SS_E_INVAL;    // not inside a block of this iteration
  *row = g.table[it->second];
  if (block_addr) *block_addr = it->first;
  return SS_OK;
}

extern "C" int ss_hook_get_stats(ss_hook_stats_t *out) {
  if (!out) return SS_E_INVAL;
  std::lock_guard<std::mutex> lock(g.mu);
  *out = g.st;
  return SS_OK;
}
