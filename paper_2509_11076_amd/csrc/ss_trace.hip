// Trace recording (Sec. 3 of the SmartSwap paper): an iteration is kept as fixed-width
// integer records, one per dispatched operator, plus the alloc/free events it caused.
// Strings (operator name, call stack) are reduced to integers once, when first seen,
// so that nothing on the per-operator path compares or hashes a string (Sec. 5.1).
// The arrays live in pinned host memory: the scan and match kernels can be fed from
// them without another staging copy.
#include <cstring>

#include "ss_internal.h"

static uint32_t fnv1a_32(const char *s) {
  uint32_t h = 0x811C9DC5u;                       // offset basis
  for (const unsigned char *p = (const unsigned char *)s; *p; ++p) {
    h ^= *p;
    h *= 0x01000193u;                             // FNV prime
  }
  return h;
}

extern "C" int ss_intern_op(ss_ctx *ctx, const char *name, const char *stack, uint32_t dtype, uint32_t n_out,
                            uint32_t phase, ss_op_t *out) {
  return ss_guard([&]() -> int {
    if (!ctx || !name || !stack || !out || dtype > 0xFF || phase > 0xFFFF) return SS_E_INVAL;
    auto it = ctx->tokens.find(name);
    uint32_t tok;
    if (it == ctx->tokens.end()) {
      tok = (uint32_t)ctx->tokens.size() + 1;       // 0 stays the padding token
      if (tok >= (1u << 18)) return SS_E_CAPACITY;  // keeps the cosine sums inside 64 bits
      ctx->tokens.emplace(name, tok);
    } else {
      tok = it->second;
    }
    auto st = ctx->stacks.find(stack);
    uint32_t h;
    if (st == ctx->stacks.end()) {
      h = fnv1a_32(stack);
      ctx->stacks.emplace(stack, h);
    } else {
      h = st->second;
    }
    out->op_token = tok;
    out->stack_hash = h;
    out->sig = (dtype & 0xFFu) | ((n_out & 0xFFu) << 8) | (phase << 16);
    out->n_out = n_out;
    return SS_OK;
  });
}

extern "C" int ss_trace_begin(ss_ctx *ctx) {
  if (!ctx) return SS_E_INVAL;
  ctx->n_ops = 0;
  ctx->n_events = 0;
  ctx->balance = 0;
  return SS_OK;
}

extern "C" int ss_trace_record(ss_ctx *ctx, const ss_op_t *op, const ss_event_t *ev, uint32_t n_ev) {
  if (!ctx || !op || (n_ev && !ev) || op->op_token == 0) return SS_E_INVAL;
  if (ctx->n_ops >= ctx->cfg.max_ops || ctx->n_events + n_ev > ctx->cfg.max_events) return SS_E_CAPACITY;
  const uint32_t idx = ctx->n_ops;
  int64_t sum = 0;
  for (uint32_t i = 0; i < n_ev; ++i) {
    if (ev[i].op_idx != idx) return SS_E_INVAL;
    sum += ev[i].delta;
  }
  ctx->ops[idx] = *op;
  if (n_ev) std::memcpy(ctx->events + ctx->n_events, ev, (size_t)n_ev * sizeof(ss_event_t));
  ctx->n_ops = idx + 1;
  ctx->n_events += n_ev;
  ctx->balance += sum;
  ctx->stats.ops_recorded++;
  ctx->stats.events_recorded += n_ev;
  return SS_OK;
}

extern "C" int ss_trace_event(ss_ctx *ctx, uint32_t tensor_id, int64_t delta) {
  if (!ctx) return SS_E_INVAL;
  if (ctx->n_ops == 0) return SS_E_ORDER;
  if (ctx->n_events >= ctx->cfg.max_events) return SS_E_CAPACITY;
  ctx->events[ctx->n_events++] = ss_event_t{ctx->n_ops - 1, tensor_id, delta};
  ctx->balance += delta;
  ctx->stats.events_recorded++;
  return SS_OK;
}

extern "C" int ss_trace_amend(ss_ctx *ctx, uint32_t op_idx, uint32_t dtype, uint32_t n_out) {
  if (!ctx || op_idx >= ctx->n_ops) return SS_E_INVAL;
  ss_op_t &o = ctx->ops[op_idx];
  o.sig = (o.sig & 0xFFFF0000u) | (dtype & 0xFFu) | ((n_out & 0xFFu) << 8);
  o.n_out = n_out;
  return SS_OK;
}

extern "C" int ss_trace_view(ss_ctx *ctx, const ss_op_t **ops, uint32_t *n_ops, const ss_event_t **ev,
                             uint64_t *n_ev, int64_t *balance) {
  if (!ctx) return SS_E_INVAL;
  if (ops) *ops = ctx->ops;
  if (n_ops) *n_ops = ctx->n_ops;
  if (ev) *ev = ctx->events;
  if (n_ev) *n_ev = ctx->n_events;
  if (balance) *balance = ctx->balance;
  return SS_OK;
}
