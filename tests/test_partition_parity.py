"""dp_partition against the oracle in oracle/partition.py: cuts, times, peaks, plans and the
search's own counters are integers and must agree exactly.  Host-only; inputs are seeded."""
import numpy as np
import pytest

import synthetic as syn
from oracle import memopt as M
from oracle import partition as P
from paper_2505_05856_amd import binding as B
from paper_2505_05856_amd.harness import to_binding_config
from test_memopt_parity import seeded_cost_model


def both(cfg, ocm, fixed_layer, fixed_stage, extra_ns=None, extra_bytes=None):
    args = (cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, cfg.micro_batch, cfg.norm_style, 2 if cfg.dtype == "bf16" else 4)
    return P.Chain(args, ocm, cfg.n_layers, fixed_layer, fixed_stage, extra_ns, extra_bytes), to_binding_config(cfg)


def same(want, got, ctx):
    assert got["feasible"] == want["feasible"], ctx
    assert got["time_ns"] == want["time_ns"], ctx
    assert got["cuts"] == want["cuts"], ctx
    assert (got["n_memopt"], got["n_positions"], got["any_memopt"]) == \
           (want["n_memopt"], want["n_positions"], want["any_memopt"]), ctx
    if "rho_cb" in want:
        assert (got["rho_cb"], got["rho_mb"]) == (want["rho_cb"], want["rho_mb"]), ctx
    for x, (w, g) in enumerate(zip(want["stages"], got["stages"])):
        for k in ("first_layer", "n_layers", "inflight", "time_ns", "base_ns", "moo_ns", "peak_bytes", "memopt"):
            assert g[k] == w[k], (ctx, x, k)
        assert list(g["plan"]) == w["plan"], (ctx, x)


CHAINS = [
    (syn.StageConfig(8, 64, 4, 256, 16, 2, "pre", True, "erf", "bf16"), 40000, 20000, None, None),
    (syn.StageConfig(8, 64, 4, 256, 16, 2, "pre", True, "erf", "bf16"), 400000, 20000, None, None),
    (syn.StageConfig(9, 64, 2, 128, 32, 1, "post", False, "erf", "bf16"), 30000, 10000,
     [90000] + [0] * 7 + [150000], [50000] + [0] * 8),
    (syn.StageConfig(7, 128, 4, 512, 16, 2, "pre", False, "tanh", "f32"), 100000, 0, None, [0, 0, 0, 300000, 0, 0, 0]),
]


@pytest.mark.parametrize("ci", range(len(CHAINS)))
@pytest.mark.parametrize("ell", [2, 3, 4, 5])
def test_partition_matches_the_oracle(ci, ell):
    cfg, fl, fs, ens, eby = CHAINS[ci]
    ocm, cm = seeded_cost_model(11 + 7 * ci, 20000, [(400, 600), (50, 50), (3000, 3000), (20, 40)][ci])
    chain, bc = both(cfg, ocm, fl, fs, ens, eby)
    loose = P.partition(chain, ell, 0)
    code, got = B.partition(bc, cm, ell, 0, fl, fs, ens, eby)
    same(loose, got, (ci, ell, "no budget"))
    need = max(s["peak_bytes"] * s["inflight"] for s in loose["stages"])
    for frac in (100, 70, 40, 15):
        budget = need * frac // 100
        want = P.partition(chain, ell, budget)
        code, got = B.partition(bc, cm, ell, budget, fl, fs, ens, eby, raise_on_error=False)
        assert (code == 0) == want["feasible"], (ci, ell, frac, B.last_error())
        if not want["feasible"]:
            assert B.STATUS[code] == "DP_E_BUDGET"
        same(want, got, (ci, ell, frac))


def test_a_single_stage_is_its_own_base_case():
    cfg = syn.StageConfig(3, 64, 4, 256, 16, 2, "pre", True, "erf", "bf16")
    ocm, cm = seeded_cost_model(5, 20000, (100, 100))
    chain, bc = both(cfg, ocm, 40000, 20000)
    need = P.partition(chain, 1, 0)["stages"][0]["peak_bytes"]
    for budget in (0, need, need * 6 // 10, need // 10):
        want = P.partition(chain, 1, budget)
        code, got = B.partition(bc, cm, 1, budget, 40000, 20000, raise_on_error=False)
        assert (code == 0) == want["feasible"]
        same(want, got, budget)


def test_balance_positions_on_benchmark_shapes():
    """The outermost rho_cb / rho_mb for chains of the benchmark layer shapes (no search cost:
    budget 0 stops at the first position)."""
    for name, n_layers, ell in (("C2", 24, 4), ("C3", 48, 8), ("C5", 32, 8)):
        import dataclasses
        cfg = dataclasses.replace(syn.CONFIGS[name], n_layers=n_layers)
        ocm, cm = seeded_cost_model(3, 10 ** 6, (50000, 50000))
        per_layer = 12 * cfg.hidden * cfg.hidden * 2 * 2
        chain, bc = both(cfg, ocm, per_layer, 4 * cfg.tokens * cfg.hidden * 2)
        want = P.partition(chain, ell, 0)
        code, got = B.partition(bc, cm, ell, 0, per_layer, 4 * cfg.tokens * cfg.hidden * 2)
        same(want, got, name)
        assert got["rho_cb"] == n_layers // 2 and got["rho_mb"] < got["rho_cb"]


def test_argument_errors():
    cfg = CHAINS[0][0]
    ocm, cm = seeded_cost_model(1, 1000, (10, 10))
    bc = to_binding_config(cfg)
    for ell in (0, 9, 33):
        code, _ = B.partition(bc, cm, ell, 0, 1, 1, raise_on_error=False)
        assert B.STATUS[code] == "DP_E_INVAL"
    code, _ = B.partition(bc, cm, 2, 0, 1, 1, extra_ns=[-1] + [0] * 7, raise_on_error=False)
    assert B.STATUS[code] == "DP_E_INVAL"
    code, out = B.partition(bc, cm, 4, 1000, 1, 1, raise_on_error=False)
    assert B.STATUS[code] == "DP_E_BUDGET" and not out["feasible"]


def test_validated_search_returns_stages_the_executor_accepts():
    """DP_MEMOPT_VALIDATE: memory is the validator's.  Every stage's plan must pass
    dp_plan_validate with the stage's in-flight count under the device budget; the model-only
    search, which does not see transient gradients and workspaces, may return one that does not."""
    import dataclasses
    cfg = syn.StageConfig(12, 128, 4, 512, 64, 2, "pre", True, "erf", "bf16")
    ocm, cm = seeded_cost_model(21, 200000, (2000, 2000))
    bc = to_binding_config(cfg)
    one = dataclasses.replace(cfg, n_layers=1)
    _, r1 = B.plan_validate(to_binding_config(one), syn.plan_keep_all(one))
    fl = r1["weight_bytes"] + r1["grad_bytes"]
    fs = r1["fixed_bytes"] - fl
    _, loose = B.partition(bc, cm, 4, 0, fl, fs, flags=B.MEMOPT_VALIDATE)
    assert loose["cuts"] == [3, 6, 9] and not loose["any_memopt"]
    need = max(s["peak_bytes"] * s["inflight"] for s in loose["stages"])
    seen_memopt = seen_moved = False
    for frac in (100, 85, 70, 55, 45):
        budget = need * frac // 100
        code, got = B.partition(bc, cm, 4, budget, fl, fs, flags=B.MEMOPT_VALIDATE, raise_on_error=False)
        if code != 0:
            assert B.STATUS[code] == "DP_E_BUDGET"
            continue
        for s in got["stages"]:
            sc = to_binding_config(dataclasses.replace(cfg, n_layers=s["n_layers"]))
            vcode, vr = B.plan_validate(sc, s["plan"], budget_bytes=budget, inflight=s["inflight"], raise_on_error=False)
            assert vcode == 0, (frac, s["first_layer"], B.last_error())
            assert s["inflight"] * vr["peak_bytes"] <= budget and vr["peak_bytes"] == s["peak_bytes"]
            assert s["time_ns"] == s["base_ns"] + s["moo_ns"]
        assert got["time_ns"] == max(s["time_ns"] for s in got["stages"])
        seen_memopt |= got["any_memopt"]
        seen_moved |= got["cuts"] != [3, 6, 9]
    assert seen_memopt and seen_moved
    code, _ = B.partition(bc, cm, 4, 0, fl, fs, flags=4, raise_on_error=False)
    assert B.STATUS[code] == "DP_E_INVAL"
