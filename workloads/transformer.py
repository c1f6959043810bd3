"""Synthetic operator/tensor traces of a stacked-decoder training iteration.

A trace is what a dispatch-point profiler would have seen in one iteration
(Sec. 3, Detailed mode): per operator a name, a call-stack string, a data type
and its output tensors; per tensor its producer, size and the operators that
use it; and the alloc/free event list of the memory trace.  Shapes follow the
paper's workload (Llama-like decoder layers stacked L times, Sec. 4.1, 6.1).

Only inputs are built here.  Tokenising the strings, scanning the memory
timeline, matching and policy timing are the method and live elsewhere.
"""
from dataclasses import dataclass, field
import numpy as np

from .layouts import (TENSOR_DT, EVENT_DT, POLICY_DT, NONE_OP, DT_BF16, DT_FP32,
                      DT_U8, DT_SIZE, PH_FWD, PH_BWD, PH_OPT)
from .rng import SplitMix64


@dataclass
class ModelShape:
    family: str          # "toy" | "flash" | "naive"
    hidden: int
    layers: int
    heads: int
    seq: int
    batch: int
    ffn_mult: int        # F = ffn_mult * hidden
    experts0: int = 0    # MoE-like extra branch ops per layer in the unperturbed trace


def config_shape(cfg):
    """Model shape of workload configuration cfg (1-based, as listed in the benchmark plan)."""
    if cfg == 1:
        return ModelShape("toy", 256, 2, 4, 128, 2, 2)
    if cfg == 2:
        return ModelShape("flash", 2048, 24, 16, 2048, 1, 4)
    if cfg in (3, 4):
        return ModelShape("naive", 4096, 32, 32, 4096, 1, 4, experts0=4 if cfg == 4 else 0)
    raise ValueError("configurations 1-4 are transformer traces; 5 is build_small_tensor_stress")


# ---- per-layer forward templates ---------------------------------------------
# op: (name, stack, inputs, outputs, gemm)   output: (tensor, size kind, dtype, saved)
# size kinds: SH = B*S*H, SF = B*S*F, S2F = B*S*2F, HSS = B*heads*S*S (elements)
# gemm: (K kind, N kind) of a dense layer computing [B*S, K] x [K, N], else None

def _layer_template(family):
    bf, u8 = DT_BF16, DT_U8
    if family == "toy":
        return [
            ("aten::layer_norm", "block.ln1", ["x"], [("ln1", "SH", bf, True)], None),
            ("aten::linear", "block.attn.q_proj", ["ln1"], [("q", "SH", bf, True)], ("H", "H")),
            ("aten::linear", "block.attn.k_proj", ["ln1"], [("k", "SH", bf, True)], ("H", "H")),
            ("aten::linear", "block.attn.v_proj", ["ln1"], [("v", "SH", bf, True)], ("H", "H")),
            ("aten::bmm", "block.attn.scores", ["q", "k"], [("scores", "HSS", bf, True)], None),
            ("aten::softmax", "block.attn.softmax", ["scores"], [("probs", "HSS", bf, True)], None),
            ("aten::bmm", "block.attn.ctx", ["probs", "v"], [("ctx", "SH", bf, True)], None),
            ("aten::linear", "block.attn.o_proj", ["ctx"], [("proj", "SH", bf, True)], ("H", "H")),
            ("aten::dropout", "block.attn.drop", ["proj"],
             [("proj_d", "SH", bf, False), ("mask", "SH", u8, True)], None),
            ("aten::add", "block.res1", ["x", "proj_d"], [("h1", "SH", bf, False)], None),
            ("aten::layer_norm", "block.ln2", ["h1"], [("ln2", "SH", bf, True)], None),
            ("aten::linear", "block.mlp.fc1", ["ln2"], [("ffn", "SF", bf, True)], ("H", "F")),
            ("aten::gelu", "block.mlp.act", ["ffn"], [("act", "SF", bf, False)], None),
            ("aten::linear", "block.mlp.fc2", ["act"], [("mlp_out", "SH", bf, True)], ("F", "H")),
            ("aten::add", "block.res2", ["h1", "mlp_out"], [("x_out", "SH", bf, False)], None),
        ]
    if family == "flash":
        return [
            ("aten::rms_norm", "block.ln1", ["x"], [("ln1", "SH", bf, True)], None),
            ("aten::linear", "block.attn.q_proj", ["ln1"], [("q", "SH", bf, True)], ("H", "H")),
            ("aten::linear", "block.attn.k_proj", ["ln1"], [("k", "SH", bf, True)], ("H", "H")),
            ("aten::linear", "block.attn.v_proj", ["ln1"], [("v", "SH", bf, True)], ("H", "H")),
            ("flash_attn::fwd", "block.attn.core", ["q", "k", "v"], [("ctx", "SH", bf, True)], ("H", "H")),
            ("aten::linear", "block.attn.o_proj", ["ctx"], [("attn_out", "SH", bf, True)], ("H", "H")),
            ("aten::add", "block.res1", ["x", "attn_out"], [("h1", "SH", bf, True)], None),
            ("aten::rms_norm", "block.ln2", ["h1"], [("ln2", "SH", bf, True)], None),
            ("aten::linear", "block.mlp.gate_up", ["ln2"], [("gu", "S2F", bf, True)], ("H", "2F")),
            ("aten::silu", "block.mlp.silu", ["gu"], [("act", "SF", bf, True)], None),
            ("aten::mul", "block.mlp.mul", ["act", "gu"], [("prod", "SF", bf, True)], None),
            ("aten::dropout", "block.mlp.drop", ["prod"],
             [("prod_d", "SF", bf, True), ("mask", "SF", u8, True)], None),
            ("aten::linear", "block.mlp.down", ["prod_d"], [("mlp_out", "SH", bf, False)], ("F", "H")),
            ("aten::add", "block.res2", ["h1", "mlp_out"], [("x_out", "SH", bf, True)], None),
        ]
    if family == "naive":
        return [
            ("aten::rms_norm", "block.ln1", ["x"], [("ln1", "SH", bf, True)], None),
            ("aten::linear", "block.attn.q_proj", ["ln1"], [("q", "SH", bf, True)], ("H", "H")),
            ("aten::linear", "block.attn.k_proj", ["ln1"], [("k", "SH", bf, True)], ("H", "H")),
            ("aten::linear", "block.attn.v_proj", ["ln1"], [("v", "SH", bf, True)], ("H", "H")),
            ("aten::bmm", "block.attn.scores", ["q", "k"], [("scores", "HSS", bf, True)], None),
            ("aten::softmax_dropout", "block.attn.softmax", ["scores"],
             [("probs", "HSS", bf, True), ("mask", "HSS", u8, True)], None),
            ("aten::bmm", "block.attn.ctx", ["probs", "v"], [("ctx", "SH", bf, True)], None),
            ("aten::linear", "block.attn.o_proj", ["ctx"], [("attn_out", "SH", bf, True)], ("H", "H")),
            ("aten::add", "block.res1", ["x", "attn_out"], [("h1", "SH", bf, True)], None),
            ("aten::rms_norm", "block.ln2", ["h1"], [("ln2", "SH", bf, True)], None),
            ("aten::linear", "block.mlp.fc1", ["ln2"], [("ffn", "SF", bf, True)], ("H", "F")),
            ("aten::gelu", "block.mlp.act", ["ffn"], [("act", "SF", bf, True)], None),
            ("aten::linear", "block.mlp.fc2", ["act"], [("mlp_out", "SH", bf, False)], ("F", "H")),
            ("aten::add", "block.res2", ["h1", "mlp_out"], [("x_out", "SH", bf, True)], None),
        ]
    raise ValueError(family)


_NOISE_OPS = ["aten::_to_copy", "aten::mul_scalar", "aten::log", "aten::isfinite",
              "aten::clamp", "aten::item", "aten::detach", "aten::view_as"]


@dataclass
class Trace:
    shape: ModelShape
    seq: int                                  # sequence length used in this iteration
    op_name: list = field(default_factory=list)
    op_stack: list = field(default_factory=list)
    op_dtype: list = field(default_factory=list)
    op_phase: list = field(default_factory=list)
    op_inputs: list = field(default_factory=list)    # tensor ids read
    op_outputs: list = field(default_factory=list)   # tensor ids written (slot order)
    op_base: list = field(default_factory=list)      # ground-truth identity, None for noise ops
    op_layer: list = field(default_factory=list)
    op_gemm: list = field(default_factory=list)      # (M, K, N) or None
    tensor_name: list = field(default_factory=list)
    tensor_layer: list = field(default_factory=list)
    tensors: np.ndarray = None                # TENSOR_DT
    events: np.ndarray = None                 # EVENT_DT, operator order, allocs before frees

    @property
    def n_ops(self):
        return len(self.op_name)


def _dim(shape, seq, kind):
    H, F = shape.hidden, shape.ffn_mult * shape.hidden
    return {"H": H, "F": F, "2F": 2 * F}[kind]


def _elems(shape, seq, kind):
    B, S, H, F = shape.batch, seq, shape.hidden, shape.ffn_mult * shape.hidden
    return {"SH": B * S * H, "SF": B * S * F, "S2F": B * S * 2 * F,
            "HSS": B * shape.heads * S * S,
            "SH8": max(1, B * S * H // 8)}[kind]


def build_trace(shape, seed=2509, iteration=0, perturb=None):
    """One iteration's trace.

    perturb = None gives the fixed sequence.  Otherwise a dict with
    p_drop, p_insert (per-operator probabilities), moe_max (per layer the
    MoE-like branch count moves by 0..moe_max around shape.experts0) and
    seq_jitter (relative sequence-length change); the random choices come from
    (seed, iteration) only.
    """
    rng = SplitMix64(seed, 1000 + iteration)
    S = shape.seq
    p_drop = p_ins = 0.0
    moe_max = 0
    if perturb:
        p_drop = perturb.get("p_drop", 0.0)
        p_ins = perturb.get("p_insert", 0.0)
        moe_max = perturb.get("moe_max", 0)
        jit = perturb.get("seq_jitter", 0.0)
        if jit:
            S = int(round(shape.seq * (1.0 + jit * (2.0 * rng.uniform() - 1.0))))
            S = max(8, (S + 7) // 8 * 8)
    tpl = _layer_template(shape.family)
    M = shape.batch * S

    # ---- 1. abstract operator list (with names of tensors) --------------------
    plan = []   # dicts: name, stack, dtype, phase, ins(names), outs[(name,kind,dt,saved)], base, layer, gemm

    def add(name, stack, phase, ins, outs, base, layer, gemm=None, dtype=DT_BF16):
        plan.append(dict(name=name, stack=stack, dtype=dtype, phase=phase, ins=list(ins),
                         outs=list(outs), base=base, layer=layer, gemm=gemm))

    add("aten::embedding", "model.embed", PH_FWD, [], [("L0.x", "SH", DT_BF16, True)],
        ("embed",), -1)
    n_exp = []
    for L in range(shape.layers):
        u = shape.experts0
        if moe_max:
            u = rng.randint(moe_max + 1)
        n_exp.append(u)
        for oi, (name, stack, ins, outs, gemm) in enumerate(tpl):
            g = None if gemm is None else (M, _dim(shape, S, gemm[0]), _dim(shape, S, gemm[1]))
            add(name, "model.layers." + stack, PH_FWD,
                ["L%d.%s" % (L, t) for t in ins],
                [("L%d.%s" % (L, t) if t != "x_out" else "L%d.x" % (L + 1), k, d, sv)
                 for (t, k, d, sv) in outs],
                ("f", L, oi), L, g)
            if stack == "block.ln2":
                for e in range(u):
                    add("aten::linear", "model.layers.block.moe.expert", PH_FWD,
                        ["L%d.ln2" % L], [("L%d.exp%d" % (L, e), "SH", DT_BF16, True)],
                        ("fe", L, e), L, (M, shape.hidden, shape.hidden))
    add("aten::cross_entropy", "model.loss", PH_FWD, ["L%d.x" % shape.layers],
        [("loss", "SH8", DT_FP32, True)], ("loss",), -1)

    fwd_plan = list(plan)
    add("aten::cross_entropy_backward", "model.loss", PH_BWD, ["loss", "L%d.x" % shape.layers],
        [("g", "SH", DT_BF16, False)], ("loss_b",), -1)
    for p in reversed(fwd_plan[1:-1]):
        saved = [t for t in p["ins"]] + [t for (t, k, d, sv) in p["outs"]]
        g = p["gemm"]
        add(p["name"] + "_backward", p["stack"], PH_BWD, ["g"] + saved,
            [("g", "SH", DT_BF16, False)], ("b",) + p["base"][1:] + (p["base"][0],), p["layer"],
            None if g is None else (g[0], g[2], g[1]))
    add("aten::embedding_backward", "model.embed", PH_BWD, ["g", "L0.x"],
        [("gw", "SH8", DT_FP32, False)], ("embed_b",), -1)
    for L in range(shape.layers):
        add("optim::adamw_step", "optimizer.step", PH_OPT, [], [], ("opt", L), L, dtype=DT_FP32)

    # ---- 2. perturb the operator list -----------------------------------------
    if p_drop or p_ins:
        out = []
        for p in plan:
            if p_ins and rng.bernoulli(p_ins):
                nm = _NOISE_OPS[rng.randint(len(_NOISE_OPS))]
                out.append(dict(name=nm, stack="train.amp.scaler", dtype=DT_FP32, phase=p["phase"],
                                ins=[], outs=[("noise", "SH8", DT_FP32, False)], base=None,
                                layer=-1, gemm=None))
            protected = p["base"] in (("embed",), ("loss",), ("loss_b",))
            if p_drop and not protected and rng.bernoulli(p_drop):
                continue
            out.append(p)
        plan = out

    # ---- 3. bind tensor names to ids, collect uses -----------------------------
    saved_names = set()
    for p in plan:
        for (t, k, d, sv) in p["outs"]:
            if sv:
                saved_names.add(t)
    tr = Trace(shape=shape, seq=S)
    live = {}          # tensor name -> id of its current instance
    rows = []          # [dtype, producer, slot, nbytes, uses(list of (op, phase))]
    for i, p in enumerate(plan):
        ins = []
        for t in p["ins"]:
            # a backward operator reads only tensors kept for it; a dropped
            # producer simply leaves the name unbound
            if t in live and (p["phase"] == PH_FWD or t == "g" or t in saved_names):
                if live[t] not in ins:
                    ins.append(live[t])
        outs = []
        for slot, (t, k, d, sv) in enumerate(p["outs"]):
            tid = len(rows)
            rows.append([d, i, slot, _elems(shape, S, k) * DT_SIZE[d], []])
            tr.tensor_name.append(t)
            tr.tensor_layer.append(p["layer"])
            live[t] = tid
            outs.append(tid)
        for tid in ins:
            rows[tid][4].append((i, p["phase"]))
        tr.op_name.append(p["name"]); tr.op_stack.append(p["stack"])
        tr.op_dtype.append(p["dtype"]); tr.op_phase.append(p["phase"])
        tr.op_inputs.append(ins); tr.op_outputs.append(outs)
        tr.op_base.append(p["base"]); tr.op_layer.append(p["layer"]); tr.op_gemm.append(p["gemm"])

    T = len(rows)
    tab = np.zeros(T, dtype=TENSOR_DT)
    for tid, (d, prod, slot, nbytes, uses) in enumerate(rows):
        fw = [o for (o, ph) in uses if ph == PH_FWD]
        bw = [o for (o, ph) in uses if ph != PH_FWD]
        in_fwd = tr.op_phase[prod] == PH_FWD
        tab[tid] = (tid, d, prod, slot, prod,
                    (max(fw) if fw else prod) if in_fwd else NONE_OP,
                    min(bw) if bw else NONE_OP,
                    max([prod] + [o for (o, _) in uses]),
                    0, 0, nbytes)
    tr.tensors = tab
    tr.events = events_of(tab)
    return tr


def events_of(tab):
    """alloc/free events of a tensor table in operator order, allocs before frees in an operator"""
    T = len(tab)
    ev = np.zeros(2 * T, dtype=EVENT_DT)
    ev["op_idx"][:T] = tab["alloc_op"]; ev["tensor_id"][:T] = tab["tensor_id"]
    ev["delta"][:T] = tab["nbytes"].astype(np.int64)
    ev["op_idx"][T:] = tab["free_op"]; ev["tensor_id"][T:] = tab["tensor_id"]
    ev["delta"][T:] = -tab["nbytes"].astype(np.int64)
    order = np.lexsort((ev["tensor_id"], ev["delta"] < 0, ev["op_idx"]))
    return ev[order]


def config_swap_set(trace, cfg):
    """The swap set a configuration prescribes outright (configurations 1 and 2).

    cfg 1: every kept-for-backward tensor of layer 0.  cfg 2: those of layers
    0, 2, 4, ...  Returned as policy rows carrying identity (producer operator,
    output slot), tensor id and size; the timing fields are left zero for the
    method to fill.
    """
    tab = trace.tensors
    lay = np.asarray(trace.tensor_layer)
    keep = ((tab["first_bwd_use"] != NONE_OP) & (tab["last_fwd_use"] != NONE_OP)
            & (tab["last_fwd_use"] < tab["first_bwd_use"]))
    if cfg == 1:
        keep &= lay == 0
    elif cfg == 2:
        keep &= (lay >= 0) & (lay % 2 == 0)
    else:
        raise ValueError("only configurations 1 and 2 prescribe the swap set")
    ids = np.nonzero(keep)[0]
    pol = np.zeros(len(ids), dtype=POLICY_DT)
    pol["ref_op"] = tab["producer_op"][ids]
    pol["out_slot"] = tab["out_slot"][ids]
    pol["tensor_id"] = ids
    pol["nbytes"] = tab["nbytes"][ids]
    return pol
