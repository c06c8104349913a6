"""CPU oracle for the pipeline partition search: the memory-balanced and compute-balanced
partitions (Appendix B.1, Algorithm 2) and the binary partition search over the positions
between them (Section 4.2, Algorithm 1: AdjacentPartition and BiPar), with the memory
optimisation of oracle/memopt.py as the MemOpt step.

TEST INFRASTRUCTURE ONLY.  Plain Python on integers (nanoseconds, bytes); nothing in the
product path imports it, it imports nothing from the product.

The model that is partitioned.  A chain of `n_layers` transformer layers of one shape (the
stage executor cuts between layers: a cut there sends exactly one [T, H] tensor to the next
stage, which is the kind of position Appendix B.2 keeps).  A layer costs the sum of its nodes'
forward and backward times (Eq. 1) plus an optional extra_ns[l] (work tied to that layer that
memory optimisation cannot touch, e.g. an embedding or an output head), and holds
fixed_per_layer + extra_bytes[l] bytes of parameters, gradients and optimiser state plus its
saved tensors.  A stage also holds fixed_per_stage bytes (its input/output buffers).

Readings of what the paper leaves open:
  * stage x of l keeps l - x + 1 micro-batches and parameter versions (Appendix B.1's ratio
    l : l-1 : ... : 1), and fits when (l - x + 1) * peak <= M (the test of Algorithm 1 line 3,
    with <= so that a budget equal to the need runs);
  * Algorithm 2's targets: M_x proportional to 1 / (l - x + 1), summing to the memory of the
    node range that is being divided (its `sum` loop and `M_x` update read that way, and it is
    what the balance equation l*M_1 = ... = M_l demands).  The walk adds a layer's memory,
    compares with the target, cuts at the layer boundary nearest to the target once it is
    reached (the paper cuts after the node that reaches it; with thousands of small nodes that
    is the same thing, with whole layers it is not) and starts the next stage from zero; nothing is released inside the forward walk (saved tensors live until the
    backward).  Targets are compared as integers through the common multiple lcm(1..l);
  * "the other partitions can be derived by adjusting Algorithm 2": the compute-balanced walk
    is the same walk over layer times with equal targets;
  * every stage keeps at least one layer: a cut is clamped so that the stages to its left and
    right still get one layer each;
  * CompMemBalPartition(N, mid, l): both walks over the node range for the stages it must
    hold; the cut after stage `mid` is rho_cb / rho_mb;
  * IdentifyAndSort: the cut positions in the closed interval between rho_cb and rho_mb,
    visited from rho_cb towards rho_mb (the early exit of both loops, "no memory optimisation
    was needed here", only makes sense in that order: further on the compute imbalance grows);
  * min(par_dict): the smallest time; ties go to the position visited first; a position where
    MemOpt cannot fit a stage into M counts as infinitely slow;
  * beyond the paper: when MemOpt fits no position of the interval into M (parameters and
    optimiser state cannot be optimised away, so condition 3 of Theorem 4.1 fails under a tight
    budget), the traversal goes on past rho_mb in the same direction (towards fewer layers in
    the earlier stages when the two coincide) and takes the first position that fits;
  * an odd number of stages: the middle is chosen so that three stages split 1 + 2 (Section 4.2:
    with three stages left the traversal starts from the first stage's positions); a single
    stage is its own base case.

Pins (tests/test_partition_oracle.py): closed forms of both walks on uniform layers, the
balance equation up to one layer, brute force over every cut vector on small chains (the search
never beats the optimum, finds it when the theorem's conditions hold, and the two-stage optimum
lies between rho_cb and rho_mb), a budget that needs no optimisation gives the compute-balanced
cuts, monotonicity in the budget, infeasibility.
"""
from __future__ import annotations

from math import lcm
from typing import Dict, List, Optional, Sequence, Tuple

from . import memopt as MO

INF = (1 << 63) - 1


class Chain:
    """The model to partition (see the module docstring)."""

    def __init__(self, layer_shape_args: Tuple, cm: MO.CostModel, n_layers: int, fixed_per_layer: int,
                 fixed_per_stage: int, extra_ns: Optional[Sequence[int]] = None,
                 extra_bytes: Optional[Sequence[int]] = None):
        # layer_shape_args: (hidden, n_heads, ffn, seq, micro_batch, style, elem_bytes[, mem_seq for style "dec"])
        self.args, self.cm, self.n = layer_shape_args, cm, int(n_layers)
        self.fixed_per_layer, self.fixed_per_stage = int(fixed_per_layer), int(fixed_per_stage)
        self.extra_ns = [int(v) for v in (extra_ns or [0] * self.n)]
        self.extra_bytes = [int(v) for v in (extra_bytes or [0] * self.n)]
        one = MO.StageShape(1, *layer_shape_args)
        self.layer_ns = sum(cm.fwd) + sum(cm.bwd)
        self.layer_saved = sum(one.bytes.values())

    def shape(self, n_layers):
        return MO.StageShape(n_layers, *self.args)

    def time_of(self, l):        # Eq. 1 over the layer's nodes
        return self.layer_ns + self.extra_ns[l]

    def mem_of(self, l):         # what the layer adds to a stage that keeps everything
        return self.fixed_per_layer + self.extra_bytes[l] + self.layer_saved


def balanced_cuts(amounts: Sequence[int], weights: Sequence[int]) -> List[int]:
    """Algorithm 2's walk.  amounts[i]: what item i adds; weights[x]: stage x's share is
    weights[x] / sum(weights) of the total.  Returns the cut after each stage but the last
    (cut c: the stage ends before item c).  The item that reaches the target closes the
    stage, unless the boundary in front of it is nearer to the target (items here are whole
    layers, not the fine-grained nodes of the paper, so the overshoot is not negligible)."""
    n, k = len(amounts), len(weights)
    assert 1 <= k <= n
    total, wsum = sum(amounts), sum(weights)
    cuts, x, cur, i, start = [], 0, 0, 0, 0
    while i < n and x < k - 1:
        a = amounts[i]
        target = total * weights[x]                 # times wsum, like everything it is compared with
        reached = (cur + a) * wsum >= target
        if reached and i > start and (cur + a) * wsum - target > target - cur * wsum:
            cuts.append(i)                          # the boundary before item i is nearer
            x, cur, start = x + 1, 0, i
            continue                                # item i opens the next stage
        cur += a
        must = n - (i + 1) == k - (x + 1)           # every later stage still needs an item
        if reached or must:
            cuts.append(i + 1)
            x, cur, start = x + 1, 0, i + 1
        i += 1
    assert len(cuts) == k - 1
    return cuts


def stage_weights(ell: int, first: int, last: int) -> List[int]:
    """Memory shares of stages first..last (1-based) of an ell-stage pipeline: 1/(ell-x+1),
    as integers over the common multiple lcm(1..ell)."""
    W = lcm(*range(1, ell + 1))
    return [W // (ell - x + 1) for x in range(first, last + 1)]


def comp_mem_bal(chain: Chain, a: int, b: int, first: int, last: int, ell: int, after: int) -> Tuple[int, int]:
    """rho_cb, rho_mb: the cut after stage `after` when layers [a, b) are divided among stages
    first..last by time and by memory (absolute layer indices)."""
    k = last - first + 1
    t = [chain.time_of(l) for l in range(a, b)]
    m = [chain.mem_of(l) for l in range(a, b)]
    cb = balanced_cuts(t, [1] * k)[after - first]
    mb = balanced_cuts(m, stage_weights(ell, first, last))[after - first]
    return a + cb, a + mb


def positions(cb: int, mb: int, lo: int, hi: int) -> Tuple[List[int], int]:
    """IdentifyAndSort: the cut positions from rho_cb to rho_mb, inside [lo, hi], and the
    direction of travel (for the continuation past rho_mb)."""
    step = 1 if mb > cb else -1
    return [p for p in range(cb, mb + step, step) if lo <= p <= hi], step


class Search:
    def __init__(self, chain: Chain, ell: int, budget: int, cache: Optional[Dict] = None):
        assert 1 <= ell <= min(chain.n, 32)
        self.c, self.ell, self.M = chain, int(ell), int(budget)
        # results of stage(); a caller may share one dict between searches of the same chain,
        # depth and budget (a stage's result is a pure function of its layers and index)
        self.cache: Dict[Tuple[int, int, int], Tuple] = {} if cache is None else cache
        self.n_memopt, self.n_positions = 0, 0

    def stage(self, a: int, b: int, x: int):
        """One stage holding layers [a, b) as stage x: (time, needed_memopt, plan, base, moo, peak).
        time = T_x + T_x^moo, INF when it cannot fit."""
        key = (a, b, x)
        if key in self.cache:
            return self.cache[key]
        n, k = b - a, self.ell - x + 1
        shape = self.c.shape(n)
        fixed = self.c.fixed_per_stage + n * self.c.fixed_per_layer + sum(self.c.extra_bytes[a:b])
        extra = sum(self.c.extra_ns[a:b])
        keep = [MO.KEEP] * (n * shape.n_slots)
        r = MO.plan_cost(shape, self.c.cm, keep, fixed)
        if self.M == 0 or k * r["peak_bytes"] <= self.M:
            out = (r["step_ns"] + extra, False, keep, r["step_ns"] + extra, 0, r["peak_bytes"])
        else:
            self.n_memopt += 1
            plan, rep = MO.memopt(shape, self.c.cm, self.M, k, fixed)
            t = rep["base_ns"] + rep["moo_ns"] + extra if rep["feasible"] else INF
            out = (t, True, plan, rep["base_ns"] + extra, rep["moo_ns"], rep["peak_bytes"])
        self.cache[key] = out
        return out

    def adjacent(self, a: int, b: int, sid: int):
        """AdjacentPartition: layers [a, b) over stages sid, sid+1.
        Returns (time of the slower stage, any memopt, [cut], [stage results])."""
        cb, mb = comp_mem_bal(self.c, a, b, sid, sid + 1, self.ell, sid)
        def at(rho):
            self.n_positions += 1
            left, right = self.stage(a, rho, sid), self.stage(rho, b, sid + 1)
            return (max(left[0], right[0]), left[1] or right[1], [rho], [left, right])
        return self.traverse(cb, mb, a + 1, b - 1, at)

    def traverse(self, cb, mb, lo, hi, at):
        """The loop both functions of Algorithm 1 share: positions from rho_cb to rho_mb, stop
        where no memory optimisation was needed, keep the fastest; if nothing fitted, go on past
        rho_mb until something does."""
        pos, step = positions(cb, mb, lo, hi)
        best = None
        for rho in pos:
            r = at(rho)
            if best is None or r[0] < best[0]:
                best = r
            if not r[1]:
                break
        if best is None or best[0] == INF:
            rho = (pos[-1] if pos else min(max(mb, lo), hi)) + step
            while lo <= rho <= hi:
                r = at(rho)
                if best is None:
                    best = r
                if r[0] < INF:
                    best = r
                    break
                rho += step
        return best

    def bipar(self, a: int, b: int, first: int, last: int):
        """BiPar over layers [a, b) and stages first..last."""
        if first == last:
            s = self.stage(a, b, first)
            return (s[0], s[1], [], [s])
        if last - first == 1:
            return self.adjacent(a, b, first)
        count = last - first + 1
        mid = first + count // 2 - 1
        cb, mb = comp_mem_bal(self.c, a, b, first, last, self.ell, mid)
        n_left, n_right = mid - first + 1, last - mid

        def at(rho):
            self.n_positions += 1
            l, r = self.bipar(a, rho, first, mid), self.bipar(rho, b, mid + 1, last)
            return (max(l[0], r[0]), l[1] or r[1], l[2] + [rho] + r[2], l[3] + r[3])
        return self.traverse(cb, mb, a + n_left, b - n_right, at)


def partition(chain: Chain, ell: int, budget: int, cache: Optional[Dict] = None):
    """BiPar(N_G, 1, l).  Returns a dict: feasible, time_ns (max over stages of T_x + T_x^moo),
    cuts (first layer of stages 2..l), stages (per stage: layers, inflight, time_ns, base_ns,
    moo_ns, peak_bytes, plan), rho_cb / rho_mb of the outermost level, counters."""
    s = Search(chain, ell, budget, cache)
    t, mopt, cuts, stages = s.bipar(0, chain.n, 1, ell)
    bounds = [0] + cuts + [chain.n]
    out = {"feasible": t < INF, "time_ns": t, "cuts": cuts, "any_memopt": mopt,
           "n_memopt": s.n_memopt, "n_positions": s.n_positions, "stages": []}
    if ell > 1:
        mid = 1 + ell // 2 - 1
        out["rho_cb"], out["rho_mb"] = comp_mem_bal(chain, 0, chain.n, 1, ell, ell, mid)
    for x, st in enumerate(stages, start=1):
        out["stages"].append({"first_layer": bounds[x - 1], "n_layers": bounds[x] - bounds[x - 1],
                              "inflight": ell - x + 1, "time_ns": st[0], "base_ns": st[3], "moo_ns": st[4],
                              "peak_bytes": st[5], "plan": list(st[2]), "memopt": st[1]})
    return out


def brute_force(chain: Chain, ell: int, budget: int, cache: Optional[Dict] = None):
    """Every cut vector, each stage optimised on its own: the true optimum of the objective
    min max_x (T_x + T_x^moo) for this MemOpt.  Small chains only."""
    from itertools import combinations
    s = Search(chain, ell, budget, cache)
    best = (INF, None)
    for cuts in combinations(range(1, chain.n), ell - 1):
        bounds = [0] + list(cuts) + [chain.n]
        t = max(s.stage(bounds[x - 1], bounds[x], x)[0] for x in range(1, ell + 1))
        if t < best[0]:
            best = (t, list(cuts))
    return best
