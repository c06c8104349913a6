"""The library's plan cost model and plan generator (dp_plan_cost, dp_plan_generate) against
the oracle in oracle/memopt.py: all quantities are integers, so everything must agree exactly.
Host-only (no GPU is needed for the planner); inputs are seeded."""
import numpy as np
import pytest

import synthetic as syn
from oracle import memopt as M
from paper_2505_05856_amd import binding as B
from paper_2505_05856_amd.harness import to_binding_config


def both_sides(cfg):
    sh = M.StageShape(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, cfg.micro_batch, cfg.norm_style,
                      2 if cfg.dtype == "bf16" else 4)
    return sh, to_binding_config(cfg)


def seeded_cost_model(seed, scale_ns, link):
    z = syn.splitmix64(seed, np.arange(16, dtype=np.uint64))
    t = [int(v % np.uint64(scale_ns)) + scale_ns // 10 for v in z]
    duplex = (max(1, link[0] * 3 // 4), max(1, link[1] * 4 // 5))     # two-way speeds, used from two in flight on
    return (M.CostModel(t[:8], t[8:], link[0], link[1], *duplex), B.make_cost_model(t[:8], t[8:], link[0], link[1], *duplex))


SMALL = [syn.StageConfig(2, 64, 4, 256, 16, 2, "pre", True, "erf", "bf16"),
         syn.StageConfig(3, 64, 2, 128, 32, 1, "post", False, "erf", "bf16"),
         syn.StageConfig(1, 128, 4, 512, 16, 2, "pre", False, "tanh", "f32"),
         syn.StageConfig(4, 64, 4, 192, 16, 3, "post", True, "erf", "f32")]


@pytest.mark.parametrize("ci", range(len(SMALL)))
def test_plan_cost_matches_the_oracle_on_random_plans(ci):
    cfg = SMALL[ci]
    sh, bc = both_sides(cfg)
    for k, link in enumerate([(1000, 1000), (50, 80), (10**9, 10**9), (7, 3)]):
        ocm, cm = seeded_cost_model(100 + 10 * ci + k, 5000, link)
        for seed in range(12):
            plan = syn.plan_seeded(cfg, 1000 * ci + seed)
            want = M.plan_cost(sh, ocm, list(plan), fixed_bytes=12345)
            got = B.plan_cost(bc, cm, plan, fixed_bytes=12345)
            assert got["step_ns"] == want["step_ns"], (ci, link, seed)
            assert got["peak_bytes"] == want["peak_bytes"]
            assert (got["d2h_bytes"], got["h2d_bytes"], got["n_replayed_ops"]) == \
                   (want["d2h_bytes"], want["h2d_bytes"], want["replayed"])
        for mk in (syn.plan_keep_all, syn.plan_all_recompute, syn.plan_all_swap):
            p = mk(cfg)
            want, got = M.plan_cost(sh, ocm, list(p)), B.plan_cost(bc, cm, p)
            assert (got["step_ns"], got["peak_bytes"]) == (want["step_ns"], want["peak_bytes"])


@pytest.mark.parametrize("ci", range(len(SMALL)))
def test_generated_plans_match_the_oracle(ci):
    cfg = SMALL[ci]
    sh, bc = both_sides(cfg)
    for k, link in enumerate([(4000, 4000), (300, 500), (20, 20)]):
        ocm, cm = seeded_cost_model(7 + 31 * ci + k, 20000, link)
        keep_peak = M.plan_cost(sh, ocm, list(syn.plan_keep_all(cfg)), fixed_bytes=4096)["peak_bytes"]
        for frac in (100, 85, 70, 55, 40, 25, 5):
            for inflight in (1, 2):
                budget = keep_peak * frac // 100 * inflight
                want_plan, want = M.memopt(sh, ocm, budget, inflight, fixed_bytes=4096)
                code, got_plan, got = B.plan_generate(bc, cm, budget, inflight, fixed_bytes=4096, raise_on_error=False)
                assert list(got_plan) == want_plan, (ci, link, frac, inflight)
                assert bool(got["feasible"]) == want["feasible"]
                assert B.STATUS[code] == ("DP_OK" if want["feasible"] else "DP_E_BUDGET")
                assert (got["base_ns"], got["moo_ns"], got["peak_bytes"]) == \
                       (want["base_ns"], want["moo_ns"], want["peak_bytes"])
                assert (got["n_free_swaps"], got["n_paid_swaps"], got["n_recomputed"]) == \
                       (want["free_swaps"], want["paid_swaps"], want["recomputed"])


def test_generate_at_workload_shapes_matches_the_oracle():
    # BERT-Large and GPT-2 stage shapes with node times and a link of the measured order of magnitude
    for name, fwd, bwd in (("C2", [37, 21, 21, 6, 35, 13, 44, 6], [11, 74, 19, 81, 11, 40, 65, 74]),
                           ("C3", [8, 300, 190, 120, 8, 380, 60, 380], [760, 70, 760, 12, 240, 520, 600, 12])):
        cfg = syn.CONFIGS[name]
        sh, bc = both_sides(cfg)
        f, b = [v * 1000 for v in fwd], [v * 1000 for v in bwd]
        ocm, cm = M.CostModel(f, b, 57000, 57000), B.make_cost_model(f, b, 57000, 57000)
        keep_peak = M.plan_cost(sh, ocm, list(syn.plan_keep_all(cfg)))["peak_bytes"]
        for frac in (80, 50):
            want_plan, want = M.memopt(sh, ocm, keep_peak * frac // 100)
            code, got_plan, got = B.plan_generate(bc, cm, keep_peak * frac // 100, raise_on_error=False)
            assert list(got_plan) == want_plan and got["moo_ns"] == want["moo_ns"], (name, frac)


def test_validated_generation_fits_the_true_peak():
    cfg = syn.CONFIGS["C3"]
    _, bc = both_sides(cfg)
    f = [8000, 300000, 190000, 120000, 8000, 380000, 60000, 380000]
    b = [760000, 70000, 760000, 12000, 240000, 520000, 600000, 12000]
    cm = B.make_cost_model(f, b, 57000, 57000)
    _, keep = B.plan_validate(bc, syn.plan_keep_all(cfg))
    _, lean = B.plan_validate(bc, syn.plan_all_recompute(cfg))
    for budget in (keep["peak_bytes"] * 9 // 10, keep["peak_bytes"] * 7 // 10, lean["peak_bytes"] * 106 // 100):
        frac = budget * 100 // keep["peak_bytes"]
        code, plan, rep = B.plan_generate(bc, cm, budget, flags=B.MEMOPT_VALIDATE, raise_on_error=False)
        assert B.STATUS[code] == "DP_OK", (frac, B.last_error())
        vcode, vrep = B.plan_validate(bc, plan, budget_bytes=budget, raise_on_error=False)
        assert B.STATUS[vcode] == "DP_OK" and vrep["peak_bytes"] <= budget
        assert rep["validated_peak_bytes"] == vrep["peak_bytes"] and rep["exact_step_ns"] >= rep["base_ns"]
    code, _, rep = B.plan_generate(bc, cm, keep["fixed_bytes"], flags=B.MEMOPT_VALIDATE, raise_on_error=False)
    assert B.STATUS[code] == "DP_E_BUDGET" and rep["feasible"] == 0


def test_argument_errors():
    cfg = SMALL[0]
    _, bc = both_sides(cfg)
    cm = B.make_cost_model([1] * 8, [1] * 8, 0, 5)
    code, _, _ = B.plan_generate(bc, cm, 0, raise_on_error=False)
    assert B.STATUS[code] == "DP_E_INVAL" and "link speed" in B.last_error()
    cm = B.make_cost_model([1] * 7 + [-1], [1] * 8, 5, 5)
    with pytest.raises(B.DpError):
        B.plan_cost(bc, cm, syn.plan_keep_all(cfg))
    cm = B.make_cost_model([1] * 8, [1] * 8, 5, 5)
    code, _, _ = B.plan_generate(bc, cm, 0, inflight=0, raise_on_error=False)
    assert B.STATUS[code] == "DP_E_INVAL"
    p = syn.plan_keep_all(cfg); p[0] = syn.RECOMPUTE
    with pytest.raises(B.DpError):
        B.plan_cost(bc, cm, p)
