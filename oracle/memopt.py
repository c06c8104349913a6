"""CPU oracle for the plan generator: the memory-optimisation step that precedes the
stage step (Section 4.3) and its cost model.

TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct Python; nothing in the
product path may import it, it imports nothing from the product and shares no code
with it.  All times are integer nanoseconds and all sizes integer bytes, so that
the product's planner can be compared with this one exactly.

What the paper fixes (Section 4.3, Section 4.2 for the objective):
  * candidates are the entries of every node's saved-tensor list;
  * they are rated by FreeTime and by memory saving per second (MSPS), the two
    quantities of the Capuchin cost model the section cites;
  * swapping is applied first, for as long as the transfers still overlap with
    computation; after that each step takes whichever of swapping or recomputation
    costs the least;
  * the result must fit the device memory (Algorithm 1's test, inflight * peak <= M)
    and the figure of merit of a stage is T_x + T_x^moo (Section 4.2).
The section only names FreeTime and MSPS; the definitions used here are those of the
cited cost model, restated:
  FreeTime(t) = (start of t's first backward use - time to copy t in)
              - (end of t's last forward use + time to copy t out),
  both taken on the timeline of the unoptimised step: the slack a swap of t has;
  MSPS(t)     = bytes saved / seconds of overhead the chosen action adds.

What the paper leaves open, and the reading taken here:
  * the timeline.  A plan's time is obtained by playing the step's schedule on three
    clocks (compute, copy-out, copy-in) with the event rules of the executor this
    planner feeds: a swap-out starts when its tensor's last forward reader is done
    and the copy-out engine is free; the swap-ins of layer l-1 are issued when the
    backward of layer l begins, each after its own copy-out has landed; a backward
    node waits for the swap-ins it reads; a recomputed tensor is regenerated on the
    compute clock right before its first backward reader by re-running its producer
    (absent inputs first), writing only outputs that are absent and still needed.
  * the memory of a plan is the running-peak walk of Algorithm 2 over the saved
    tensors (add at allocation, take the maximum, subtract at release) plus a fixed
    part passed in by the caller; a swapped-out tensor is released when its copy-out
    has landed (seen from the compute clock at the next allocation), not when the
    copy is queued.
  * "until the transfers no longer overlap": candidates are visited by decreasing
    FreeTime and the first one whose swap lengthens the step ends the phase.
  * the second phase repeatedly takes, over all remaining candidates and both
    actions, the one with the largest MSPS among those that lower the peak; when no
    single change lowers it (two moments share the peak) it takes, among the changes
    that do not raise it, the one with the most tensor bytes per second of overhead.

Pins (tests/test_memopt_oracle.py): closed forms of the timeline (keep-all, all
recompute, infinite and tiny link speed), a hand-worked two-layer example stored
under tests/golden/, the peak of keep-all by hand, brute force over all plans of a
one-layer stage, monotonicity in the budget.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

KEEP, RECOMPUTE, SWAP = 0, 1, 2
SLOTS = ("X_IN", "LN1_STATS", "LN1_OUT", "QKV", "ATTN_LSE", "ATTN_OUT",
         "RES1", "LN2_STATS", "LN2_OUT", "FC1_OUT", "GELU_OUT", "RES2")
# a decoder layer (style "dec": the pre-LN layer with a cross-attention block over an encoder
# memory between its attention and its feed-forward block) saves seven more tensors
CROSS_SLOTS = ("LNC_STATS", "LNC_OUT", "Q_C", "KV_C", "ATTN_C_LSE", "ATTN_C_OUT", "RES_C")
SLOT = {n: i for i, n in enumerate(SLOTS + CROSS_SLOTS)}
N_SLOTS = len(SLOTS)

# Forward nodes of one layer in execution order: (name, inputs, outputs); "NEXT" is the
# layer's output, which is the next layer's X_IN.
_FWD = {
    "pre": [("LN1", ["X_IN"], ["LN1_OUT", "LN1_STATS"]),
            ("QKV", ["LN1_OUT"], ["QKV"]),
            ("ATTN", ["QKV"], ["ATTN_OUT", "ATTN_LSE"]),
            ("PROJ", ["ATTN_OUT", "X_IN"], ["RES1"]),
            ("LN2", ["RES1"], ["LN2_OUT", "LN2_STATS"]),
            ("FC1", ["LN2_OUT"], ["FC1_OUT"]),
            ("GELU", ["FC1_OUT"], ["GELU_OUT"]),
            ("FC2", ["GELU_OUT", "RES1"], ["NEXT"])],
    "post": [("QKV", ["X_IN"], ["QKV"]),
             ("ATTN", ["QKV"], ["ATTN_OUT", "ATTN_LSE"]),
             ("PROJ", ["ATTN_OUT", "X_IN"], ["RES1"]),
             ("LN1", ["RES1"], ["LN1_OUT", "LN1_STATS"]),
             ("FC1", ["LN1_OUT"], ["FC1_OUT"]),
             ("GELU", ["FC1_OUT"], ["GELU_OUT"]),
             ("FC2", ["GELU_OUT", "LN1_OUT"], ["RES2"]),
             ("LN2", ["RES2"], ["NEXT", "LN2_STATS"])],
    # the key/value projection reads the encoder memory, which is not a saved tensor
    "dec": [("LN1", ["X_IN"], ["LN1_OUT", "LN1_STATS"]),
            ("QKV", ["LN1_OUT"], ["QKV"]),
            ("ATTN", ["QKV"], ["ATTN_OUT", "ATTN_LSE"]),
            ("PROJ", ["ATTN_OUT", "X_IN"], ["RES1"]),
            ("LNC", ["RES1"], ["LNC_OUT", "LNC_STATS"]),
            ("QC", ["LNC_OUT"], ["Q_C"]),
            ("KVC", [], ["KV_C"]),
            ("ATTNC", ["Q_C", "KV_C"], ["ATTN_C_OUT", "ATTN_C_LSE"]),
            ("PROJC", ["ATTN_C_OUT", "RES1"], ["RES_C"]),
            ("LN2", ["RES_C"], ["LN2_OUT", "LN2_STATS"]),
            ("FC1", ["LN2_OUT"], ["FC1_OUT"]),
            ("GELU", ["FC1_OUT"], ["GELU_OUT"]),
            ("FC2", ["GELU_OUT", "RES_C"], ["NEXT"])],
}
# Backward nodes of one layer in execution order: (name, saved tensors read, saved tensors
# released when the node is done).
_BWD = {
    "pre": [("FC2", ["GELU_OUT"], ["GELU_OUT"]),
            ("GELU", ["FC1_OUT"], ["FC1_OUT"]),
            ("FC1", ["LN2_OUT"], ["LN2_OUT"]),
            ("LN2", ["RES1", "LN2_STATS"], ["RES1", "LN2_STATS"]),
            ("PROJ", ["ATTN_OUT"], []),
            ("ATTN", ["QKV", "ATTN_OUT", "ATTN_LSE"], ["QKV", "ATTN_OUT", "ATTN_LSE"]),
            ("QKV", ["LN1_OUT"], ["LN1_OUT"]),
            ("LN1", ["X_IN", "LN1_STATS"], ["X_IN", "LN1_STATS"])],
    "post": [("LN2", ["RES2", "LN2_STATS"], ["RES2", "LN2_STATS"]),
             ("FC2", ["GELU_OUT"], ["GELU_OUT"]),
             ("GELU", ["FC1_OUT"], ["FC1_OUT"]),
             ("FC1", ["LN1_OUT"], ["LN1_OUT"]),
             ("LN1", ["RES1", "LN1_STATS"], ["RES1", "LN1_STATS"]),
             ("PROJ", ["ATTN_OUT"], []),
             ("ATTN", ["QKV", "ATTN_OUT", "ATTN_LSE"], ["QKV", "ATTN_OUT", "ATTN_LSE"]),
             ("QKV", ["X_IN"], ["X_IN"])],
    "dec": [("FC2", ["GELU_OUT"], ["GELU_OUT"]),
            ("GELU", ["FC1_OUT"], ["FC1_OUT"]),
            ("FC1", ["LN2_OUT"], ["LN2_OUT"]),
            ("LN2", ["RES_C", "LN2_STATS"], ["RES_C", "LN2_STATS"]),
            ("PROJC", ["ATTN_C_OUT"], []),
            ("ATTNC", ["Q_C", "KV_C", "ATTN_C_LSE"], ["Q_C", "KV_C", "ATTN_C_OUT", "ATTN_C_LSE"]),
            ("KVC", [], []),
            ("QC", ["LNC_OUT"], ["LNC_OUT"]),
            ("LNC", ["RES1", "LNC_STATS"], ["RES1", "LNC_STATS"]),
            ("PROJ", ["ATTN_OUT"], []),
            ("ATTN", ["QKV", "ATTN_OUT", "ATTN_LSE"], ["QKV", "ATTN_OUT", "ATTN_LSE"]),
            ("QKV", ["LN1_OUT"], ["LN1_OUT"]),
            ("LN1", ["X_IN", "LN1_STATS"], ["X_IN", "LN1_STATS"])],
}


class StageShape:
    """Sizes of the saved tensors of one layer.  T = micro_batch * seq tokens."""

    def __init__(self, n_layers, hidden, n_heads, ffn, seq, micro_batch, style, elem_bytes, mem_seq=0):
        self.L, self.style = int(n_layers), style
        assert (style == "dec") == (mem_seq > 0)
        self.slots = SLOTS + CROSS_SLOTS if style == "dec" else SLOTS
        self.n_slots = len(self.slots)
        T, H, F = micro_batch * seq, hidden, ffn
        e = elem_bytes
        self.bytes = {"X_IN": T * H * e, "LN1_STATS": T * 2 * 4, "LN1_OUT": T * H * e, "QKV": T * 3 * H * e,
                      "ATTN_LSE": micro_batch * n_heads * seq * 4, "ATTN_OUT": T * H * e, "RES1": T * H * e,
                      "LN2_STATS": T * 2 * 4, "LN2_OUT": T * H * e, "FC1_OUT": T * F * e, "GELU_OUT": T * F * e,
                      "RES2": T * H * e}
        # the slot that is only another name of the next layer's input has no storage
        self.bytes["RES2" if style in ("pre", "dec") else "LN2_OUT"] = 0
        if style == "dec":
            Tm = micro_batch * mem_seq
            self.bytes.update({"LNC_STATS": T * 2 * 4, "LNC_OUT": T * H * e, "Q_C": T * H * e, "KV_C": Tm * 2 * H * e,
                               "ATTN_C_LSE": micro_batch * n_heads * seq * 4, "ATTN_C_OUT": T * H * e,
                               "RES_C": T * H * e})

    def has_storage(self, name):
        return self.bytes[name] > 0


class CostModel:
    """fwd_ns[i], bwd_ns[i]: time of the i-th forward / backward node of a layer (execution
    order of the style); d2h, h2d: link speed in bytes per microsecond."""

    def __init__(self, fwd_ns: Sequence[int], bwd_ns: Sequence[int], d2h_bytes_per_us: int, h2d_bytes_per_us: int,
                 d2h_duplex: int = 0, h2d_duplex: int = 0):
        assert len(fwd_ns) == len(bwd_ns) and len(fwd_ns) in (8, 13)      # thirteen nodes: a decoder layer
        self.fwd, self.bwd = [int(v) for v in fwd_ns], [int(v) for v in bwd_ns]
        self.d2h, self.h2d = int(d2h_bytes_per_us), int(h2d_bytes_per_us)
        # link speed with both directions busy (0: not known)
        self.d2h_duplex, self.h2d_duplex = int(d2h_duplex), int(h2d_duplex)

    def for_inflight(self, inflight: int) -> "CostModel":
        """The model a planner uses for a stage with `inflight` micro-batches between forward and
        backward: from two on, copy-outs of one micro-batch and copy-ins of another run side by
        side all the time, so the two-way link speed applies where it is known."""
        if inflight < 2:
            return self
        return CostModel(self.fwd, self.bwd, self.d2h_duplex or self.d2h, self.h2d_duplex or self.h2d,
                         self.d2h_duplex, self.h2d_duplex)

    def out_ns(self, nbytes):
        return -((-nbytes * 1000) // self.d2h)      # ceiling

    def in_ns(self, nbytes):
        return -((-nbytes * 1000) // self.h2d)


def _where_lives(l, name):
    return (l + 1, "X_IN") if name == "NEXT" else (l, name)


def plan_cost(shape: StageShape, cm: CostModel, plan, fixed_bytes: int = 0) -> Dict[str, int]:
    """Plays one step under `plan` ([L * shape.n_slots] actions).  Returns step_ns, peak_bytes (fixed +
    running peak of the saved tensors), d2h_bytes, h2d_bytes, replayed (nodes re-run)."""
    L, fwd, bwd = shape.L, _FWD[shape.style], _BWD[shape.style]
    SLOTS, N_SLOTS = shape.slots, shape.n_slots
    assert len(cm.fwd) == len(fwd)

    def action(l, name):
        if l >= L or not shape.has_storage(name) or (name == "X_IN" and l == 0):
            return KEEP
        return int(plan[l * N_SLOTS + SLOT[name]])

    def owned(l, name):     # the library holds it (the stage input and output are the caller's)
        return not (name == "X_IN" and (l == 0 or l == L))

    clk = {"c": 0, "out": 0, "in": 0}
    where: Dict[Tuple[int, str], str] = {(0, "X_IN"): "dev"}
    consumed = set()
    out_done: Dict[Tuple[int, str], int] = {}
    ready: Dict[Tuple[int, str], int] = {}
    live = peak = 0
    stats = {"d2h_bytes": 0, "h2d_bytes": 0, "replayed": 0}

    lingering: List[Tuple[int, int]] = []      # (time its copy-out lands, bytes) of swapped-out tensors

    def settle():
        nonlocal live
        for item in [x for x in lingering if x[0] <= clk["c"]]:
            live -= item[1]
            lingering.remove(item)

    def alloc(key):
        nonlocal live, peak
        settle()
        if owned(*key):
            live += shape.bytes[key[1]]
            peak = max(peak, live)
        where[key] = "dev"

    def free(key):
        nonlocal live
        if where.get(key) != "dev":
            return
        if key in ready:                       # a copy-in may still be in flight into it
            clk["c"] = max(clk["c"], ready.pop(key))
        if owned(*key):
            live -= shape.bytes[key[1]]
        del where[key]

    def swap_out(key):
        nonlocal live
        start = max(clk["out"], clk["c"])
        clk["out"] = start + cm.out_ns(shape.bytes[key[1]])
        out_done[key] = clk["out"]
        stats["d2h_bytes"] += shape.bytes[key[1]]
        lingering.append((clk["out"], shape.bytes[key[1]]))   # its memory is reusable once the copy has landed
        where[key] = "host"

    def swap_in(key):
        if where.get(key) != "host":
            return
        alloc(key)
        start = max(clk["in"], clk["c"], out_done[key])
        clk["in"] = start + cm.in_ns(shape.bytes[key[1]])
        ready[key] = clk["in"]
        stats["h2d_bytes"] += shape.bytes[key[1]]

    # ---- forward
    for l in range(L):
        last = {}
        for i, (_, ins, outs) in enumerate(fwd):
            for n in ins + outs:
                if n != "NEXT":
                    last[n] = i
        for i, (_, ins, outs) in enumerate(fwd):
            for n in outs:
                alloc(_where_lives(l, n))
            clk["c"] += cm.fwd[i]
            for n in SLOTS:                    # in slot order
                if last.get(n) != i or where.get((l, n)) != "dev":
                    continue
                a = action(l, n)
                if a == RECOMPUTE:
                    free((l, n))
                elif a == SWAP:
                    swap_out((l, n))

    # ---- backward
    def ensure(l, name):
        key = (l, name)
        if where.get(key) == "host":
            swap_in(key)
        if where.get(key) == "dev":
            if key in ready:
                clk["c"] = max(clk["c"], ready.pop(key))
            return
        pl, target = (l - 1, "NEXT") if name == "X_IN" else (l, name)
        for i, (_, ins, outs) in enumerate(fwd):
            if target in outs:
                for n in ins:
                    ensure(pl, n)
                for n in outs:
                    k2 = _where_lives(pl, n)
                    if k2 not in where and k2 not in consumed:
                        alloc(k2)
                clk["c"] += cm.fwd[i]
                stats["replayed"] += 1
                return
        raise KeyError(name)

    def prefetch(l):
        """The swap-ins of layer l, in the order its backward first reads them."""
        if l >= 0:
            for _, reads, _ in bwd:
                for n in reads:
                    swap_in((l, n))        # (a second call finds the tensor on the device)
            for n in SLOTS:                # whatever no backward node reads
                swap_in((l, n))

    prefetch(L - 1)
    for l in reversed(range(L)):
        prefetch(l - 1)
        for i, (_, reads, releases) in enumerate(bwd):
            for n in reads:
                ensure(l, n)
            clk["c"] += cm.bwd[i]
            for n in releases:
                free((l, n))
                consumed.add((l, n))
        for n in SLOTS:                        # whatever a replay left behind in this layer
            free((l, n))
            consumed.add((l, n))
    step = max(clk["c"], clk["out"], clk["in"])
    return {"step_ns": step, "peak_bytes": fixed_bytes + peak, **stats}


def candidates(shape: StageShape) -> List[Tuple[int, str]]:
    return [(l, n) for l in range(shape.L) for n in shape.slots
            if shape.has_storage(n) and not (l == 0 and n == "X_IN")]


def free_times(shape: StageShape, cm: CostModel) -> Dict[Tuple[int, str], int]:
    """FreeTime of every candidate on the timeline of the unoptimised step."""
    L, fwd, bwd = shape.L, _FWD[shape.style], _BWD[shape.style]
    t = 0
    last_use_end: Dict[Tuple[int, str], int] = {}
    for l in range(L):
        for i, (_, ins, outs) in enumerate(fwd):
            t += cm.fwd[i]
            for n in ins + outs:
                last_use_end[_where_lives(l, n)] = t
    first_use_start: Dict[Tuple[int, str], int] = {}
    for l in reversed(range(L)):
        for i, (_, reads, _rel) in enumerate(bwd):
            for n in reads:
                first_use_start.setdefault((l, n), t)
            t += cm.bwd[i]
    ft = {}
    for key in candidates(shape):
        b = shape.bytes[key[1]]
        ft[key] = (first_use_start[key] - cm.in_ns(b)) - (last_use_end[key] + cm.out_ns(b))
    return ft


def memopt(shape: StageShape, cm: CostModel, budget_bytes: int, inflight: int = 1, fixed_bytes: int = 0):
    """The two phases of Section 4.3.  Returns (plan, report); report has feasible, base_ns
    (T_x: the unoptimised step), moo_ns (T_x^moo: what the plan adds), peak_bytes, and the
    number of tensors swapped for free, swapped at a cost and recomputed."""
    L, N_SLOTS = shape.L, shape.n_slots
    plan = [KEEP] * (L * N_SLOTS)
    cm = cm.for_inflight(inflight)

    def cost(p):
        r = plan_cost(shape, cm, p, fixed_bytes)
        return r["step_ns"], r["peak_bytes"]

    def fits(peak):
        return budget_bytes == 0 or inflight * peak <= budget_bytes

    def idx(key):
        return key[0] * N_SLOTS + SLOT[key[1]]

    T, P = cost(plan)
    base = T
    ft = free_times(shape, cm)
    order = sorted(candidates(shape), key=lambda k: (-ft[k], k[0], SLOT[k[1]]))
    counts = {"free_swaps": 0, "paid_swaps": 0, "recomputed": 0}
    # phase 1: swaps for as long as they still hide behind computation
    for key in order:
        if fits(P):
            break
        trial = list(plan)
        trial[idx(key)] = SWAP
        T1, P1 = cost(trial)
        if T1 > T:
            break
        plan, T, P = trial, T1, P1
        counts["free_swaps"] += 1
    # phase 2: the action with the most memory saved per second of overhead
    rest = [k for k in order if plan[idx(k)] == KEEP]
    while not fits(P):
        best = None
        for plateau in (False, True):
            for pos, key in enumerate(rest):
                for a in (SWAP, RECOMPUTE):
                    trial = list(plan)
                    trial[idx(key)] = a
                    T1, P1 = cost(trial)
                    dt = max(T1 - T, 0)
                    # first pass: changes that lower the peak, rated by the peak reduction;
                    # second pass (none found): changes that keep it, rated by the tensor's size
                    if (P1 >= P) if not plateau else (P1 > P):
                        continue
                    saved = P - P1 if not plateau else shape.bytes[key[1]]
                    # larger saved/(dt+1) wins; then smaller dt; then swap before recompute; then order
                    if best is None:
                        better = True
                    else:
                        lhs, rhs = saved * (best["dt"] + 1), best["saved"] * (dt + 1)
                        better = lhs > rhs or (lhs == rhs and dt < best["dt"])
                    if better:
                        best = {"pos": pos, "key": key, "a": a, "saved": saved, "dt": dt, "T": T1, "P": P1}
            if best is not None:
                break
        if best is None:
            return plan, {"feasible": False, "base_ns": base, "moo_ns": T - base, "peak_bytes": P, **counts}
        plan[idx(best["key"])] = best["a"]
        T, P = best["T"], best["P"]
        counts["paid_swaps" if best["a"] == SWAP else "recomputed"] += 1
        rest.pop(best["pos"])
    return plan, {"feasible": True, "base_ns": base, "moo_ns": T - base, "peak_bytes": P, **counts}
