"""Overhead of the online profiler hook on a real PyTorch training step (the comparison of the
paper's profiler-overhead table, Sec. 6: no profiling, Lightweight mode, Detailed mode, and
PyTorch's built-in profiler), on one GPU.

    python -m paper_2509_11076_amd.hook_overhead [--layers 12 --hidden 1024 --seq 1024 --batch 4]

The model is a small Llama-like decoder written in plain PyTorch with random weights and random token
ids; one step = zero_grad, forward, loss, backward, AdamW step.  Prints one JSON line.
"""
import argparse
import json
import sys
import time

import torch
import torch.nn as nn
import torch.nn.functional as F


class Block(nn.Module):
    def __init__(self, hidden, heads, ffn):
        super().__init__()
        self.heads = heads
        self.ln1 = nn.RMSNorm(hidden)
        self.qkv = nn.Linear(hidden, 3 * hidden, bias=False)
        self.o = nn.Linear(hidden, hidden, bias=False)
        self.ln2 = nn.RMSNorm(hidden)
        self.gate_up = nn.Linear(hidden, 2 * ffn, bias=False)
        self.down = nn.Linear(ffn, hidden, bias=False)

    def forward(self, x):
        b, s, h = x.shape
        q, k, v = self.qkv(self.ln1(x)).view(b, s, 3, self.heads, h // self.heads).permute(2, 0, 3, 1, 4)
        a = F.scaled_dot_product_attention(q, k, v, is_causal=True)
        x = x + self.o(a.transpose(1, 2).reshape(b, s, h))
        g, u = self.gate_up(self.ln2(x)).chunk(2, dim=-1)
        return x + self.down(F.silu(g) * u)


class Decoder(nn.Module):
    def __init__(self, vocab, hidden, layers, heads, ffn):
        super().__init__()
        self.embed = nn.Embedding(vocab, hidden)
        self.blocks = nn.ModuleList([Block(hidden, heads, ffn) for _ in range(layers)])
        self.norm = nn.RMSNorm(hidden)
        self.head = nn.Linear(hidden, vocab, bias=False)

    def forward(self, ids):
        x = self.embed(ids)
        for blk in self.blocks:
            x = blk(x)
        return self.head(self.norm(x))


class Trainer:
    """One training step with the phase announced to the hook (when one is given)."""

    def __init__(self, args, device="cuda"):
        torch.manual_seed(2509)
        self.model = Decoder(args.vocab, args.hidden, args.layers, args.heads, 4 * args.hidden).to(
            device=device, dtype=torch.bfloat16)
        self.opt = torch.optim.AdamW(self.model.parameters(), lr=1e-4)
        g = torch.Generator(device="cpu").manual_seed(11)
        self.ids = torch.randint(0, args.vocab, (args.batch, args.seq), generator=g).to(device)
        self.tgt = torch.randint(0, args.vocab, (args.batch, args.seq), generator=g).to(device)
        self.hook = None

    def step(self):
        H = self.hook
        self.opt.zero_grad(set_to_none=True)
        if H:
            H.ss_hook_begin_iteration()
        logits = self.model(self.ids)
        loss = F.cross_entropy(logits.view(-1, logits.shape[-1]).float(), self.tgt.view(-1))
        if H:
            H.ss_hook_set_phase(1)
        loss.backward()
        if H:
            H.ss_hook_set_phase(2)
        self.opt.step()
        return loss


def timed(fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    t_host = time.perf_counter() - t0
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3, t_host / steps * 1e3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=12)
    ap.add_argument("--hidden", type=int, default=1024)
    ap.add_argument("--heads", type=int, default=16)
    ap.add_argument("--seq", type=int, default=1024)
    ap.add_argument("--batch", type=int, default=4)
    ap.add_argument("--vocab", type=int, default=32000)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    args = ap.parse_args()
    from . import binding as B
    from . import torch_hook as H

    torch.cuda.set_device(0)
    tr = Trainer(args)
    rows = {}

    def report(name, ms, host_ms, extra=None):
        rows[name] = dict(ms_per_step=round(ms, 3), host_ms_per_step=round(host_ms, 3), **(extra or {}))
        print("%-28s %.3f ms/step (host %.3f)" % (name, ms, host_ms), file=sys.stderr, flush=True)

    ms, host = timed(tr.step, args.steps, args.warmup)
    report("no profiling", ms, host)

    cfg = B.ss_config_default()
    cfg.staging_bytes = 4096
    cfg.max_ops = 1 << 18
    cfg.max_events = 1 << 20
    ctx = B.ss_create(cfg)
    tr.hook = H
    try:
        for name, mode in (("hook, Lightweight mode", H.SS_HOOK_LIGHTWEIGHT), ("hook, Detailed mode", H.SS_HOOK_DETAILED)):
            H.ss_hook_install(ctx, mode)
            ms, host = timed(tr.step, args.steps, args.warmup)
            ops, ev, bal = B.ss_trace_view(ctx)
            report(name, ms, host, dict(ops_per_step=len(ops), events_per_step=len(ev),
                                        distinct_operators=int(len(set(ops["op_token"].tolist())))))
        H.ss_hook_set_mode(H.SS_HOOK_OFF)
        ms, host = timed(tr.step, args.steps, args.warmup)
        report("hook installed, switched off", ms, host)
    finally:
        H.ss_hook_remove()
        tr.hook = None
        B.ss_destroy(ctx)

    from torch.profiler import profile, ProfilerActivity
    for name, kw in (("torch.profiler, CPU activity", dict()),
                     ("torch.profiler, shapes+memory+stacks", dict(record_shapes=True, profile_memory=True,
                                                                     with_stack=True))):
        for _ in range(2):
            tr.step()
        torch.cuda.synchronize()
        n = max(3, args.steps // 4)
        with profile(activities=[ProfilerActivity.CPU], **kw):
            ms, host = timed(tr.step, n, 1)
        report(name, ms, host, dict(steps=n))

    base = rows["no profiling"]["ms_per_step"]
    for r in rows.values():
        r["overhead_pct"] = round(100 * (r["ms_per_step"] / base - 1), 1)
    print(json.dumps({"workload": "Llama-like decoder, %d layers, hidden %d, %d heads, seq %d, batch %d, bf16, AdamW"
                                  % (args.layers, args.hidden, args.heads, args.seq, args.batch),
                      "steps": args.steps, "warmup": args.warmup, "modes": rows}), flush=True)


if __name__ == "__main__":
    main()
