"""Pins for the partition-search oracle (Algorithm 2's balance walks, Algorithm 1's
AdjacentPartition / BiPar): closed forms, the balance equation, Theorem 4.1 on two stages,
brute force over every cut vector, behaviour in the budget."""
import itertools

import pytest

from oracle import memopt as MO
from oracle import partition as P

CM = MO.CostModel([10, 30, 20, 10, 10, 40, 10, 40], [40, 12, 40, 15, 20, 45, 60, 15], 50, 50)
LAYER = (64, 2, 256, 32, 2, "pre", 2)      # hidden, heads, ffn, seq, micro-batch, style, bytes per element


def chain(n, fixed_layer=400000, fixed_stage=20000, style="pre", **kw):
    return P.Chain(LAYER[:5] + (style,) + LAYER[6:], CM, n, fixed_layer, fixed_stage, **kw)


# ---------------------------------------------------------------- the balance walks
def test_compute_balance_of_uniform_layers_is_equal_counts():
    for n, k in [(8, 4), (12, 3), (6, 2), (5, 5)]:
        assert P.balanced_cuts([7] * n, [1] * k) == [n // k * (x + 1) for x in range(k - 1)]


def test_memory_balance_follows_the_pipedream_ratio():
    """Two stages: stage 1 keeps two micro-batches, so it gets a third of the memory; four
    stages: shares 1/4 : 1/3 : 1/2 : 1 of lcm 12 = 3 : 4 : 6 : 12 of 25."""
    assert P.stage_weights(2, 1, 2) == [1, 2] and P.stage_weights(4, 1, 4) == [3, 4, 6, 12]
    assert P.stage_weights(4, 3, 4) == [6, 12]                  # a sub-range keeps the global depths
    assert P.balanced_cuts([1] * 6, [1, 2]) == [2]
    assert P.balanced_cuts([1] * 25, [3, 4, 6, 12]) == [3, 7, 13]


@pytest.mark.parametrize("n,ell", [(24, 2), (48, 4), (60, 5), (64, 8)])
def test_balance_equation_holds_to_one_layer(n, ell):
    """(l - x + 1) * M_x is the same for every stage, up to the granularity of one layer."""
    amounts = [100 + (7 * i) % 13 for i in range(n)]
    cuts = P.balanced_cuts(amounts, P.stage_weights(ell, 1, ell))
    bounds = [0] + cuts + [n]
    held = [(ell - x) * sum(amounts[bounds[x]:bounds[x + 1]]) for x in range(ell)]
    assert max(held) - min(held) <= ell * max(amounts) * 2
    assert all(b > a for a, b in zip(bounds, bounds[1:]))


def test_every_stage_keeps_a_layer_and_the_nearest_boundary_is_taken():
    assert P.balanced_cuts([5, 1, 1, 1], [1, 1, 1, 1]) == [1, 2, 3]
    assert P.balanced_cuts([1, 1, 1, 9], [1, 1]) == [3]
    assert P.balanced_cuts([9, 1, 1, 1], [1, 1]) == [1]
    # 6 reaches the target 5 by overshooting 1, stopping before it would miss by 2: after it
    assert P.balanced_cuts([3, 3, 4], [1, 1]) == [2]
    # 7 overshoots the target 4 by 3, stopping before it misses by 1: before it
    assert P.balanced_cuts([3, 4, 1], [1, 1]) == [1]


def test_positions_run_from_rho_cb_to_rho_mb():
    assert P.positions(6, 3, 1, 9) == ([6, 5, 4, 3], -1)
    assert P.positions(3, 6, 4, 9) == ([4, 5, 6], 1)
    assert P.positions(5, 5, 1, 9) == ([5], -1)


# ---------------------------------------------------------------- the search
def test_a_budget_that_needs_no_optimisation_gives_the_compute_balanced_cuts():
    ch = chain(8)
    r = P.partition(ch, 4, 0)
    assert r["cuts"] == [2, 4, 6] and not r["any_memopt"] and r["n_memopt"] == 0
    assert r["time_ns"] == 2 * ch.layer_ns                      # Eq. 1: two layers a stage
    assert [s["inflight"] for s in r["stages"]] == [4, 3, 2, 1]
    assert r["n_positions"] == 3                                # one position per level pair: the early exit


def test_two_stage_optimum_lies_between_the_balanced_positions():
    """Theorem 4.1 on a uniform chain (its three conditions hold), over budgets from loose to
    tight: the brute-force optimum's cut is in [rho_mb, rho_cb] and the search finds its time."""
    ch = chain(7, fixed_layer=40000)
    for M in (0, 2 * 10 ** 6, 1200000, 900000):
        memo = {}
        r = P.partition(ch, 2, M, memo)
        t, cuts = P.brute_force(ch, 2, M, memo)
        if t == P.INF:
            assert not r["feasible"]
            continue
        lo, hi = sorted((r["rho_cb"], r["rho_mb"]))
        assert r["time_ns"] == t
        # among the cuts that reach the optimum one lies in the interval
        s = P.Search(ch, 2, M, memo)
        optimal = [c for c in range(1, ch.n) if max(s.stage(0, c, 1)[0], s.stage(c, ch.n, 2)[0]) == t]
        assert any(lo <= c <= hi for c in optimal), (M, optimal, lo, hi)


CASES = [(chain(6), 4), (chain(7, fixed_layer=40000), 4), (chain(6, fixed_layer=40000), 3),
         (chain(7, 40000, 20000, "post", extra_ns=[300] + [0] * 5 + [500], extra_bytes=[10 ** 5] + [0] * 6), 4),
         (chain(5, fixed_layer=100000), 2), (chain(4, fixed_layer=100000), 1)]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_against_brute_force_over_every_cut_vector(case):
    ch, ell = CASES[case]
    loose = P.partition(ch, ell, 0)
    peak = max(s["peak_bytes"] * s["inflight"] for s in loose["stages"])
    seen_memopt = False
    for frac in (1.0, 0.85, 0.65, 0.45):
        M = int(peak * frac)
        memo = {}
        r = P.partition(ch, ell, M, memo)
        t, cuts = P.brute_force(ch, ell, M, memo)
        assert r["time_ns"] >= t                                   # never better than the optimum
        if t < P.INF:
            assert r["feasible"], (frac, cuts)
            assert r["time_ns"] == t, (frac, r["cuts"], cuts)      # and on these chains it finds it
            assert all(s["inflight"] * s["peak_bytes"] <= M for s in r["stages"])
            bounds = [0] + r["cuts"] + [ch.n]
            assert [s["n_layers"] for s in r["stages"]] == [b - a for a, b in zip(bounds, bounds[1:])]
            assert r["time_ns"] == max(s["time_ns"] for s in r["stages"])
            assert all(s["time_ns"] == s["base_ns"] + s["moo_ns"] for s in r["stages"])
            seen_memopt |= r["any_memopt"]
    assert seen_memopt or case in (0, 5)        # (parameters dominate case 0: nothing to optimise away)


def test_time_is_monotone_in_the_budget_and_a_hopeless_budget_is_reported():
    ch = chain(8, fixed_layer=40000)
    last = 0
    for M in (4 * 10 ** 6, 2 * 10 ** 6, 1500000, 1200000, 10 ** 6, 800000):
        r = P.partition(ch, 4, M)
        if r["feasible"]:
            assert r["time_ns"] >= last
            last = r["time_ns"]
    r = P.partition(ch, 4, 1000)
    assert not r["feasible"] and r["time_ns"] == P.INF


def test_three_stages_split_one_plus_two_and_extras_move_the_cuts():
    ch = chain(9, fixed_layer=40000)
    s = P.Search(ch, 3, 0)
    seen = []
    orig = s.adjacent
    s.adjacent = lambda a, b, sid: (seen.append((a, b, sid)), orig(a, b, sid))[1]
    s.bipar(0, 9, 1, 3)
    assert seen and all(sid == 2 for _, _, sid in seen)          # stages 2 and 3 form the adjacent pair
    plain = P.partition(ch, 3, 0)["cuts"]
    heavy_head = P.partition(chain(9, fixed_layer=40000, extra_ns=[0] * 8 + [3 * ch.layer_ns]), 3, 0)["cuts"]
    assert plain == [3, 6] and heavy_head[-1] > plain[-1]         # the last stage gives up layers
