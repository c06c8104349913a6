"""Pins of the plan-generator oracle (oracle/memopt.py) against closed forms, a hand-worked
example, brute force and invariants.  CPU only."""
import itertools
import os

import pytest

from oracle import memopt as M

F = [10, 20, 30, 40, 50, 60, 70, 80]
Bk = [15, 25, 35, 45, 55, 65, 75, 85]
HERE = os.path.dirname(os.path.abspath(__file__))


def shape(L=1, style="pre"):
    return M.StageShape(L, 64, 4, 256, 16, 2, style, 2)


def plan_with(sh, actions):
    p = [M.KEEP] * (sh.L * M.N_SLOTS)
    for (l, name), a in actions.items():
        p[l * M.N_SLOTS + M.SLOT[name]] = a
    return p


def test_worked_example_from_golden_file():
    want = {}
    for line in open(os.path.join(HERE, "golden", "memopt_worked_example.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            want[k] = int(v)
    sh = shape(1, "pre")
    cm = M.CostModel(F, Bk, 102400, 61440)
    got = M.plan_cost(sh, cm, plan_with(sh, {(0, "QKV"): M.SWAP, (0, "LN2_OUT"): M.RECOMPUTE}))
    for k in ("step_ns", "peak_bytes", "d2h_bytes", "h2d_bytes", "replayed"):
        assert got[k] == want[k], k
    assert M.plan_cost(sh, cm, plan_with(sh, {}))["step_ns"] == want["base_ns"]


@pytest.mark.parametrize("style", ["pre", "post"])
@pytest.mark.parametrize("L", [1, 3])
def test_keep_all_closed_forms(style, L):
    sh = shape(L, style)
    r = M.plan_cost(sh, M.CostModel(F, Bk, 1000, 1000), plan_with(sh, {}), fixed_bytes=777)
    assert r["step_ns"] == L * (sum(F) + sum(Bk))
    # every saved tensor of every layer is alive when forward ends; the inputs of layers 1.. are the library's
    per_layer = sum(v for n, v in sh.bytes.items() if n != "X_IN")
    assert r["peak_bytes"] == 777 + L * per_layer + (L - 1) * sh.bytes["X_IN"]
    assert r["d2h_bytes"] == r["h2d_bytes"] == r["replayed"] == 0


@pytest.mark.parametrize("style", ["pre", "post"])
def test_recomputing_one_tensor_adds_its_producer_and_frees_it_in_the_lower_layers(style):
    L = 3
    sh = shape(L, style)
    cm = M.CostModel(F, Bk, 1000, 1000)
    base = M.plan_cost(sh, cm, plan_with(sh, {}))
    gelu_node = [n for n, _, _ in M._FWD[style]].index("GELU")
    r = M.plan_cost(sh, cm, plan_with(sh, {(l, "GELU_OUT"): M.RECOMPUTE for l in range(L)}))
    assert r["step_ns"] == base["step_ns"] + L * F[gelu_node]
    assert r["replayed"] == L
    # pre-LN: the top layer's GELU_OUT is alive with everything else (forward: until FC2, the last node, is
    # done; backward: regenerated first).  post-LN: it goes when FC2 is done, before the last node (LN2)
    # allocates its statistics, and comes back after LN2's backward has released them.
    late = 0 if style == "pre" else sh.bytes["LN2_STATS"]
    assert r["peak_bytes"] == base["peak_bytes"] - (L - 1) * sh.bytes["GELU_OUT"] - late


def test_all_recompute_replays_every_node_once():
    # every saved tensor dropped (the inputs of layers 1.. too): backward re-runs each forward node once.
    # pre-LN: except the top layer's last node, which only produces the stage output; post-LN's last node
    # (LN2) also produces statistics its own backward reads, so it is re-run too.
    for style in ("pre", "post"):
        L = 2
        sh = shape(L, style)
        cm = M.CostModel(F, Bk, 1000, 1000)
        p = [M.RECOMPUTE] * (L * M.N_SLOTS)
        r = M.plan_cost(sh, cm, p)
        skipped = 1 if style == "pre" else 0
        assert r["replayed"] == 8 * L - skipped
        assert r["step_ns"] == L * (sum(F) + sum(Bk)) + L * sum(F) - skipped * F[7]


def test_swap_is_free_on_a_fast_link_and_serial_on_a_slow_one():
    L = 2
    sh = shape(L, "pre")
    base = L * (sum(F) + sum(Bk))
    p = plan_with(sh, {(L - 1, "GELU_OUT"): M.SWAP})
    fast = M.plan_cost(sh, M.CostModel(F, Bk, 10**12, 10**12), p)
    assert fast["step_ns"] == base + 2 and fast["d2h_bytes"] == sh.bytes["GELU_OUT"]   # 1 ns each way, on the critical path
    hidden = M.plan_cost(sh, M.CostModel(F, Bk, 10**5, 10**5), plan_with(sh, {(0, "LN1_OUT"): M.SWAP}))
    assert hidden["step_ns"] == base            # 41 ns each way, between its uses there are more than 1000 ns
    # slow link: GELU_OUT of the top layer is last read by the last forward node and first needed by the
    # first backward node, so the step is forward + copy-out + copy-in + backward
    slow = M.CostModel(F, Bk, 4, 8)
    r = M.plan_cost(sh, slow, p)
    assert r["step_ns"] == base + slow.out_ns(sh.bytes["GELU_OUT"]) + slow.in_ns(sh.bytes["GELU_OUT"])
    assert slow.out_ns(16384) == 4096000 and slow.in_ns(16384) == 2048000


def test_free_time_definition():
    sh = shape(2, "pre")
    cm = M.CostModel(F, Bk, 1000, 500)
    ft = M.free_times(sh, cm)
    Tf, Tb = sum(F), sum(Bk)
    # LN1_OUT of layer 0: last forward reader QKV (ends at 30); first backward reader is the QKV node of
    # layer 0, which starts after the whole backward of layer 1 and the first six nodes of layer 0
    first = 2 * Tf + Tb + sum(Bk[:6])
    b = sh.bytes["LN1_OUT"]
    assert ft[(0, "LN1_OUT")] == (first - cm.in_ns(b)) - (30 + cm.out_ns(b))
    # the input of layer 1 is last read by layer 1's PROJ and first needed by layer 1's LN1 (last node)
    b = sh.bytes["X_IN"]
    assert ft[(1, "X_IN")] == (2 * Tf + sum(Bk[:7]) - cm.in_ns(b)) - (Tf + sum(F[:4]) + cm.out_ns(b))
    assert (0, "X_IN") not in ft and (0, "RES2") not in ft


def _brute_force(sh, cm):
    cands = M.candidates(sh)
    out = []
    for acts in itertools.product((M.KEEP, M.RECOMPUTE, M.SWAP), repeat=len(cands)):
        p = plan_with(sh, dict(zip(cands, acts)))
        r = M.plan_cost(sh, cm, p)
        out.append((r["peak_bytes"], r["step_ns"]))
    return out


def test_generated_plans_against_brute_force_on_one_layer():
    sh = shape(1, "post")
    cm = M.CostModel([40, 30, 20, 10, 60, 10, 60, 10], [20, 100, 20, 100, 20, 40, 60, 70], 200000, 200000)
    every = _brute_force(sh, cm)           # 3^10 plans
    keep_peak = M.plan_cost(sh, cm, plan_with(sh, {}))["peak_bytes"]
    base = M.plan_cost(sh, cm, plan_with(sh, {}))["step_ns"]
    smallest = min(p for p, _ in every)
    for budget in (keep_peak, keep_peak * 3 // 4, keep_peak // 2, smallest, smallest - 1):
        plan, rep = M.memopt(sh, cm, budget)
        r = M.plan_cost(sh, cm, plan)
        optimum = min((t for p, t in every if p <= budget), default=None)
        assert rep["base_ns"] == base and rep["moo_ns"] == r["step_ns"] - base and rep["peak_bytes"] == r["peak_bytes"]
        if rep["feasible"]:
            assert r["peak_bytes"] <= budget
            assert optimum is not None and optimum <= r["step_ns"]
            # the greedy is not optimal in general; on this stage it stays within 5 % of the best plan
            assert r["step_ns"] <= optimum * 1.05
        else:
            assert r["peak_bytes"] > budget
    assert M.memopt(sh, cm, smallest - 1)[1]["feasible"] is False
    assert M.memopt(sh, cm, keep_peak)[1]["moo_ns"] == 0


def test_phase_one_swaps_cost_nothing_and_budget_is_monotone():
    sh = shape(3, "pre")
    cm = M.CostModel([5000 * v for v in F], [5000 * v for v in Bk], 50000, 50000)
    keep_peak = M.plan_cost(sh, cm, plan_with(sh, {}))["peak_bytes"]
    prev = None
    for frac in (100, 90, 80, 70, 60, 50, 40):
        plan, rep = M.memopt(sh, cm, keep_peak * frac // 100)
        if not rep["feasible"]:
            break
        if rep["paid_swaps"] == 0 and rep["recomputed"] == 0:
            assert rep["moo_ns"] == 0          # only hidden swaps so far
        if prev is not None:
            assert rep["moo_ns"] >= prev       # a tighter budget never makes the plan cheaper
        prev = rep["moo_ns"]
    assert prev is not None


def test_inflight_multiplies_the_peak():
    sh = shape(2, "pre")
    cm = M.CostModel(F, Bk, 1000, 1000)
    keep_peak = M.plan_cost(sh, cm, plan_with(sh, {}))["peak_bytes"]
    assert M.memopt(sh, cm, keep_peak, inflight=1)[1]["moo_ns"] == 0
    plan, rep = M.memopt(sh, cm, keep_peak, inflight=2)
    assert (not rep["feasible"]) or 2 * rep["peak_bytes"] <= keep_peak


def test_two_way_link_speed_applies_from_two_micro_batches_in_flight():
    """A stage that keeps two micro-batches in flight plans with the two-way link speed (its copy-outs and
    copy-ins overlap all the time); one in flight, or no two-way figure, plans with the one-way speed."""
    sh = M.StageShape(2, 64, 2, 256, 32, 2, "pre", 2)
    f, b = [10, 30, 20, 10, 10, 40, 10, 40], [40, 12, 40, 15, 20, 45, 60, 15]
    fast, slow = M.CostModel(f, b, 40000, 40000), M.CostModel(f, b, 100, 150)
    both = M.CostModel(f, b, 40000, 40000, 100, 150)
    keep = M.plan_cost(sh, fast, [M.KEEP] * (2 * M.N_SLOTS))["peak_bytes"]
    budget = keep * 6 // 10
    assert M.memopt(sh, both, budget, 1) == M.memopt(sh, fast, budget, 1)
    assert M.memopt(sh, both, 2 * budget, 2) == M.memopt(sh, slow, 2 * budget, 2)
    # the fast link hides five swaps behind the computation, the two-way speed hides none
    assert M.memopt(sh, both, 2 * budget, 2)[1]["free_swaps"] < M.memopt(sh, fast, 2 * budget, 2)[1]["free_swaps"]
    assert both.for_inflight(1) is both and both.for_inflight(3).d2h == 100 and fast.for_inflight(3).h2d == 40000
