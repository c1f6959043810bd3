"""Synthetic compute stream: stand-in for the training step the swaps overlap with.

Every operator of a generated trace is given device work of the matching kind
on the compute stream: dense layers run bf16 GEMMs of the model's shapes
(forward into the activation tensors themselves; backward as two GEMMs of the
same cost on scratch buffers), other operators run element-wise kernels over
their tensors.  Backward operators read every tensor kept for them: an exact
integer checksum of its bytes is recorded and its values are folded into the
gradient, so that a tensor that came back late, wrong, or into memory someone
else still used changes the results.  All of it is plain PyTorch (hipBLASLt
GEMMs, element-wise kernels); none of it is the swap path.
"""
import numpy as np
import torch

from .layouts import DT_BF16, DT_FP32, DT_U8, PH_FWD, NONE_OP

_TORCH_DT = {DT_BF16: torch.bfloat16, DT_FP32: torch.float32, DT_U8: torch.uint8}


class SyntheticCompute:
    def __init__(self, trace, arena, seed=2509, gemm_scale=1.0):
        """arena: 1-D uint8 CUDA tensor that holds every tensor of `trace` at its dev_off
        (and, after a swap-in, at dev_off_in).  gemm_scale < 1 shrinks the GEMM K dimension
        (for quick tests)."""
        self.tr = trace
        self.arena = arena
        dev = arena.device
        g = torch.Generator(device=dev)
        g.manual_seed(seed)
        tab = trace.tensors
        self.fwd_view, self.bwd_view = [], []
        for t in tab:
            dt = _TORCH_DT[int(t["dtype"])]
            n = int(t["nbytes"])
            a = arena[int(t["dev_off"]):int(t["dev_off"]) + n].view(dt)
            b = arena[int(t["dev_off_in"]):int(t["dev_off_in"]) + n].view(dt)
            self.fwd_view.append(a)
            self.bwd_view.append(b)
        self.swapped = set()
        # weights per distinct dense-layer shape, small values so activations stay finite
        self.weights = {}
        max_m = max_k = max_n = 1
        for gm in trace.op_gemm:
            if gm is None:
                continue
            M, K, N = gm
            K = max(16, int(K * gemm_scale))
            max_m, max_k, max_n = max(max_m, M), max(max_k, K), max(max_n, N)
            if (K, N) not in self.weights:
                w = torch.randn(K, N, generator=g, device=dev, dtype=torch.float32) * (1.0 / K ** 0.5)
                self.weights[(K, N)] = w.to(torch.bfloat16)
        self.gemm_scale = gemm_scale
        # scratch operands of the backward GEMMs (cost only)
        self.scr_a = (torch.randn(max_m * max(max_k, max_n), generator=g, device=dev) * 0.1).to(torch.bfloat16)
        self.scr_o = torch.empty(max_m * max(max_k, max_n), device=dev, dtype=torch.bfloat16)
        self.checksum = torch.zeros(len(tab), dtype=torch.int64, device=dev)
        self.x0 = torch.randn(int(tab["nbytes"][0]) // 2, generator=g, device=dev).to(torch.bfloat16)

    def mark_swapped(self, tensor_ids):
        """tensors whose backward-side address is dev_off_in"""
        self.swapped = set(int(t) for t in tensor_ids)

    def _view(self, tid, phase):
        if phase != PH_FWD and tid in self.swapped:
            return self.bwd_view[tid]
        return self.fwd_view[tid]

    @staticmethod
    def _spread(dst, src):
        """define every element of dst from src (flat), whatever the two sizes and types are"""
        dst = dst.view(-1)
        src = src.view(-1)
        if dst.dtype == torch.uint8 and src.dtype != torch.uint8:
            src = src.view(torch.uint8)
        n, m = dst.numel(), src.numel()
        if n <= m:
            dst.copy_(src[:n])
        elif n % m == 0:
            dst.view(n // m, m).copy_(src.view(1, m).expand(n // m, m))
        else:
            r = n // m
            dst[:r * m].view(r, m).copy_(src.view(1, m).expand(r, m))
            dst[r * m:].copy_(src[:n - r * m])

    def run_op(self, i):
        tr = self.tr
        phase = tr.op_phase[i]
        ins = [self._view(t, phase) for t in tr.op_inputs[i]]
        outs = [self._view(t, phase) for t in tr.op_outputs[i] if t is not None]
        gm = tr.op_gemm[i]
        if phase == PH_FWD:
            if not ins:                                    # embedding: the iteration's input
                for o in outs:
                    self._spread(o, self.x0)
                return
            if gm is not None and outs and outs[0].dtype == torch.bfloat16 and ins[0].dtype == torch.bfloat16:
                M, K, N = gm
                Kc = max(16, int(K * self.gemm_scale))
                a = ins[0].view(-1)
                if a.numel() >= M * K and outs[0].numel() == M * N:
                    torch.mm(a[:M * K].view(M, K)[:, :Kc], self.weights[(Kc, N)], out=outs[0].view(M, N))
                    for o in outs[1:]:
                        self._spread(o, ins[0])
                    return
            for k, o in enumerate(outs):
                self._spread(o, ins[min(k, len(ins) - 1)])
                if o.dtype == torch.bfloat16 and len(ins) > 1 and k == 0:
                    other = ins[1].view(-1)
                    if other.dtype == torch.bfloat16:
                        n = min(o.numel(), other.numel())
                        o.view(-1)[:n].add_(other[:n], alpha=0.5)
            return
        # backward / optimizer
        if gm is not None:
            M, Kb, Nb = gm                                  # backward of a forward [M, Nb] x [Nb, Kb]
            Kc = max(16, int(Nb * self.gemm_scale))
            w = self.weights.get((Kc, Kb))
            if w is not None:
                for _ in range(2):                         # grad-input and grad-weight GEMMs (cost only)
                    torch.mm(self.scr_a[:M * Kc].view(M, Kc), w, out=self.scr_o[:M * Kb].view(M, Kb))
        if not outs:
            return
        g_out = outs[0]
        grad_in = None
        for t, v in zip(tr.op_inputs[i], ins):
            if tr.tensor_name[t] == "g":
                grad_in = v
            else:
                # exact integer checksum of every byte of the kept tensor
                nb = v.numel() * v.element_size()
                raw = v.view(-1).view(torch.uint8)
                n4 = nb // 4 * 4
                s = raw[:n4].view(torch.int32).sum(dtype=torch.int64)
                if n4 < nb:
                    s = s + raw[n4:].sum(dtype=torch.int64)
                self.checksum[t] += s * (i + 1)
        if grad_in is not None:
            self._spread(g_out, grad_in)
            if g_out.dtype == torch.bfloat16:
                g_out.view(-1).mul_(0.5)
        else:
            self._spread(g_out, self.x0)
        for t, v in zip(tr.op_inputs[i], ins):
            if tr.tensor_name[t] != "g" and v.dtype == torch.bfloat16 and g_out.dtype == torch.bfloat16:
                n = min(v.numel(), g_out.numel())
                g_out.view(-1)[:n].add_(v.view(-1)[:n], alpha=0.125)

    def result(self):
        """what must be bit-identical with and without swapping: checksums of every kept tensor as
        its backward operators saw it, and the last gradient"""
        tr = self.tr
        last = None
        for i in range(tr.n_ops - 1, -1, -1):
            if tr.op_outputs[i] and tr.op_phase[i] != PH_FWD:
                last = self._view(tr.op_outputs[i][0], tr.op_phase[i])
                break
        torch.cuda.synchronize()
        return self.checksum.cpu().numpy().copy(), (last.view(-1).view(torch.uint8).cpu().numpy().copy()
                                                    if last is not None else np.zeros(0, np.uint8))
