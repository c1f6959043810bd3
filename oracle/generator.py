"""Policy generator of Sec. 4 (test oracle): logical layers, memory reduction list, candidate
list with the score of Eq. 2, the swap simulator, and the loop of Algo. 2.

Steps follow the paper's order and notation.  What it leaves open is fixed as follows (each is
this build's reading; the paper prints no worked example, so the pins are a case worked by hand from
its steps, the order Eq. 2 prescribes, invariants and brute force):

 * Time is counted in link bytes, so Eq. 3 (T_swap = S / B) makes T_swap = S and Eq. 1
   (T_group = T_iter / N_iter * N_group) makes a layer's time budget bpo * N_group with
   bpo = B * T_iter / N_iter.  Everything stays in integers.  Optionally bpo is given per phase
   (B * T_phase / N_phase): Eq. 1 applied to the forward, backward and optimizer operators
   separately, for hardware on which a forward operator is several times shorter than a backward one.
 * Logical layers (Sec. 4.1, 4.3): the forward operators, in execution order, are cut into
   g_fwd groups of (almost) equal operator count, group g taking positions
   [g * n // G, (g + 1) * n // G); the backward operators likewise into g_bwd groups; all
   optimizer operators form one layer.  A layer records its first operator, one past its last,
   its type and T_remaining; swap-ins and swap-outs draw on the same T_remaining.
 * MRL (Sec. 4.2): one entry per operator whose memory without swaps exceeds the limit, holding
   the excess.
 * CL (Sec. 4.2): tensors kept from forward to backward (last forward use < first backward use),
   not smaller than min_bytes, not yet in the policy, with N_MRE > 0, where N_MRE is the number
   of MRL entries at operators t with last forward use + 1 < t < first backward use (the block
   can be released after the operator that follows the last forward use at the earliest, so
   these are the entries the tensor can be away from).
   Score = N_MRE / max N_MRE + C * S / max S over the list (Eq. 2) with C = c_num / c_den,
   compared exactly as N_MRE * maxS * c_den + c_num * S * maxN; ties: larger tensor, lower id.
 * Swap-in (Sec. 4.3.1): candidates in descending score.  A candidate that no longer spans any
   MRL entry is skipped.  Let L_use be the layer of the first backward use and L_peak the layer
   of the last MRL entry the tensor still spans.  The search runs over L = L_use - 1 down to
   L_peak + 1 for T_remaining(L) > S ("before the peak memory period": a swap-in placed at or
   before L_peak would bring the tensor back while memory is still over the limit).  The
   swap-in is issued before the first operator of the layer found.  A candidate without such a
   layer is passed over; if the whole list is passed over, the highest-scoring candidate that
   still spans an entry is scheduled in layer L_use - 1 regardless of T_remaining (flag LATE).
   Committing a candidate subtracts S from the layer's T_remaining and S from every MRL entry at
   an operator t with last forward use + 1 < t < swap-in operator (entries reaching 0 vanish).
 * Algo. 2: repeat {build CL; empty -> error; simulate} until the MRL is empty.
 * SetFreeTime (Sec. 4.3.2): items in swap-out order (last forward use, then tensor id).  From
   the layer of the last forward use forward to the layer before the swap-in layer, the first
   layer with T_remaining > S takes the swap-out; none -> the layer before the swap-in layer
   (flag LATE).  The swap-out is triggered right after the last forward use (Sec. 4.3.2, first
   sentence), so of that use's own layer only the operators that follow the use can carry it:
   there the test is min(T_remaining, bpo * operators of the layer after the use) > S.  The
   block is released after the last operator of the layer found (Sec. 5.2), but never before
   the operator after the last forward use.
"""
NONE_OP = 0xFFFFFFFF
F_LATE = 4


class Infeasible(Exception):
    pass


def logical_layers(phases, g_fwd, g_bwd, bpo):
    """phases: per operator 0 forward / 1 backward / 2 optimizer.  Returns (layers, layer_of) with
    layers = list of dicts(first, end, type, remaining) in operator order and layer_of[op].
    bpo: link bytes per operator, one number (Eq. 1 as printed: the iteration time spread evenly
    over all operators) or three, one per phase (Eq. 1 applied to each phase's own measured time)."""
    n = len(phases)
    bpo3 = tuple(int(b) for b in bpo) if isinstance(bpo, (tuple, list)) else (int(bpo),) * 3
    layers = []
    for ph, G in ((0, g_fwd), (1, g_bwd), (2, 1)):
        idx = [i for i in range(n) if phases[i] == ph]
        if not idx:
            continue
        G = max(1, min(G, len(idx)))
        for g in range(G):
            lo, hi = g * len(idx) // G, (g + 1) * len(idx) // G
            if hi > lo:
                layers.append(dict(first=idx[lo], end=idx[hi - 1] + 1, type=ph,
                                   remaining=bpo3[ph] * (hi - lo), ops=idx[lo:hi], bpo=bpo3[ph]))
    layers.sort(key=lambda L: L["first"])
    layer_of = [0] * n
    for li, L in enumerate(layers):
        for i in L["ops"]:
            layer_of[i] = li
    return layers, layer_of


def generate_policy(tensors, per_op_memory, phases, limit, bpo, g_fwd, g_bwd, c_num=1, c_den=1, min_bytes=0):
    """Algo. 2.  per_op_memory[t] = memory in use at operator t without swaps (from the timeline
    scan).  Returns (items, info): items are tuples
    (ref_op, out_slot, tensor_id, flags, t_out, t_free, t_in, t_use, nbytes) in the order they were
    committed; info has the per-round candidate lists and the residual MRL (empty on success)."""
    n = len(phases)
    layers, layer_of = logical_layers(phases, g_fwd, g_bwd, bpo)
    mrl = {t: int(per_op_memory[t]) - int(limit) for t in range(n) if int(per_op_memory[t]) > int(limit)}
    chosen = {}
    rounds = []

    def spans(t):
        lf, fb = int(t["last_fwd_use"]), int(t["first_bwd_use"])
        return [op for op in mrl if lf + 1 < op < fb]

    while mrl:
        # ---- candidate list with Eq. 2
        cl = []
        for t in tensors:
            lf, fb, S = int(t["last_fwd_use"]), int(t["first_bwd_use"]), int(t["nbytes"])
            if lf == NONE_OP or fb == NONE_OP or not lf < fb or S < min_bytes or int(t["tensor_id"]) in chosen:
                continue
            n_mre = len(spans(t))
            if n_mre > 0:
                cl.append((t, n_mre, S))
        if not cl:
            raise Infeasible("memory reduction list not empty and no candidate left")
        max_n = max(c[1] for c in cl)
        max_s = max(c[2] for c in cl)
        cl.sort(key=lambda c: (-(c[1] * max_s * c_den + c_num * c[2] * max_n), -c[2], int(c[0]["tensor_id"])))
        rounds.append([int(c[0]["tensor_id"]) for c in cl])

        # ---- simulate: pre-trigger swap-in
        def commit(t, L_in, late):
            lf, fb, S = int(t["last_fwd_use"]), int(t["first_bwd_use"]), int(t["nbytes"])
            t_in = layers[L_in]["first"]
            layers[L_in]["remaining"] -= S
            for op in [op for op in mrl if lf + 1 < op < t_in]:
                mrl[op] -= S
                if mrl[op] <= 0:
                    del mrl[op]
            chosen[int(t["tensor_id"])] = dict(t=t, L_in=L_in, t_in=t_in, late=late)

        committed = 0
        for (t, _, S) in cl:
            if not mrl:
                break
            sp = spans(t)
            if not sp:
                continue
            L_use = layer_of[int(t["first_bwd_use"])]
            L_peak = layer_of[max(sp)]
            for L in range(L_use - 1, L_peak, -1):
                if layers[L]["remaining"] > S:
                    commit(t, L, False)
                    committed += 1
                    break
        if committed == 0 and mrl:
            for (t, _, S) in cl:                       # fallback: accept latency rather than stop
                if spans(t):
                    L_use = layer_of[int(t["first_bwd_use"])]
                    L_in = max(L_use - 1, layer_of[int(t["last_fwd_use"])] + 1)
                    if L_in > L_use:
                        continue
                    commit(t, L_in, True)
                    committed += 1
                    break
            if committed == 0:
                raise Infeasible("no candidate can be scheduled")

    # ---- SetFreeTime: swap-out completion
    order = sorted(chosen.values(), key=lambda c: (int(c["t"]["last_fwd_use"]), int(c["t"]["tensor_id"])))
    for c in order:
        t = c["t"]
        lf, S = int(t["last_fwd_use"]), int(t["nbytes"])
        L0 = layer_of[lf]
        last = c["L_in"] - 1
        found = None
        for L in range(L0, last + 1):
            avail = layers[L]["remaining"]
            if L == L0:                        # only what follows the last forward use within its own layer
                avail = min(avail, layers[L]["bpo"] * sum(1 for op in layers[L]["ops"] if op > lf))
            if avail > S:
                found = L
                break
        if found is None:
            found = max(L0, last)
            c["late"] = True
        layers[found]["remaining"] -= S
        c["t_free"] = min(max(layers[found]["end"] - 1, lf + 1), c["t_in"] - 1)
    items = []
    for tid, c in chosen.items():
        t = c["t"]
        items.append((int(t["producer_op"]), int(t["out_slot"]), tid, F_LATE if c["late"] else 0,
                      int(t["last_fwd_use"]), c["t_free"], c["t_in"], int(t["first_bwd_use"]), int(t["nbytes"])))
    return items, dict(rounds=rounds, residual=dict(mrl),
                       layers=[(L["first"], L["end"], L["type"], L["remaining"]) for L in layers])


def generate_policy_best(tensors, events, n_ops, base, phases, limit, bpo, param_sets):
    """Several parameter sets (dicts g_fwd, g_bwd, c_num, c_den, min_bytes): one policy each, each
    scanned with its own points, the best kept: no operator over the limit first (else fewest such
    operators), then fewest LATE items, then fewest bytes, then the lowest index.  Infeasible sets
    are skipped.  Returns (items, chosen index, dict(peak, n_over, n_late, bytes))."""
    from .timeline import timeline_scan
    mem = timeline_scan(events, None, n_ops, base, limit)["per_op"]
    best = None
    for c, p in enumerate(param_sets):
        per_phase = tuple(int(b) or int(bpo) for b in p.get("phase_bytes_per_op") or (0, 0, 0))
        try:
            items, _ = generate_policy(tensors, mem, phases, limit, per_phase, p["g_fwd"], p["g_bwd"],
                                       p.get("c_num", 1), p.get("c_den", 1), p.get("min_bytes", 0))
        except Infeasible:
            continue
        pe = []
        for it in items:
            pe += [(it[5], it[2], -it[8]), (it[6], it[2], it[8])]
        pe.sort(key=lambda e: e[0])
        sc = timeline_scan(events, pe, n_ops, base, limit)
        key = (sc["n_over"], sum(1 for it in items if it[3] & F_LATE), sum(it[8] for it in items), c)
        if best is None or key < best[0]:
            best = (key, items, c, sc)
    if best is None:
        raise Infeasible("every parameter set runs out of candidates")
    key, items, c, sc = best
    return items, c, dict(peak=sc["peak"], n_over=key[0], n_late=key[1], bytes=key[2])
