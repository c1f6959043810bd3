"""A small Llama-like decoder in plain PyTorch with a one-call training step (harness plumbing).

Stands in for the "real model" the dispatch hook of libss_torch_hook.so is exercised on: random
weights, random token ids; one step = zero_grad, forward, loss, backward, AdamW step, with the phase
announced to the hook when one is attached.  Nothing of the method lives here.
"""
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
        self.saved_hooks = None      # optional: a context-manager factory around forward + backward (autograd's
                                     # saved-tensor hooks), and callbacks at the phase changes
        self.on_phase = None

    def step(self):
        import contextlib
        H = self.hook
        self.opt.zero_grad(set_to_none=True)
        if H:
            H.ss_hook_begin_iteration()
        with (self.saved_hooks() if self.saved_hooks else contextlib.nullcontext()):
            logits = self.model(self.ids)
            loss = F.cross_entropy(logits.view(-1, logits.shape[-1]).float(), self.tgt.view(-1))
            if H:
                H.ss_hook_set_phase(1)
            if self.on_phase:
                self.on_phase(1)
            loss.backward()
        if H:
            H.ss_hook_set_phase(2)
        if self.on_phase:
            self.on_phase(2)
        self.opt.step()
        if self.on_phase:
            self.on_phase(3)
        return loss
