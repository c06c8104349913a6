"""Plan generator against the device: a cost model measured on this GPU, plans generated
for shrinking budgets, each run through dp_stage_step: it must fit its budget, give the
bits of the all-KEEP step.  Predicted against measured times are printed; the assertions on
them only catch a gross disagreement (a factor of two): the box's clocks move with the data
and the load, and a wall-clock tolerance must not decide whether the parity results after it
in the run are seen."""
import time

import pytest
import torch

import synthetic as syn
from paper_2505_05856_amd import binding as B
from paper_2505_05856_amd.harness import StageRunner

pytestmark = pytest.mark.gpu


def timed(run, plan, budget, n=8):
    for _ in range(2):
        run.step(plan, budget)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        run.step(plan, budget)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / n * 1e9


@pytest.mark.parametrize("name", ["C3", "C2"])
def test_generated_plans_fit_run_and_match_the_prediction(name):
    cfg = syn.CONFIGS[name]
    run = StageRunner(cfg, syn.make_weights(cfg), *syn.make_activations(cfg))
    keep = syn.plan_keep_all(cfg)
    run.step(keep, 0)
    want_bits = run.raw_results()
    cm = B.stage_measure_cost_model(run.stage, run.x, run.dy, run.y, run.dx, run.g, steps=3)
    d = cm.as_dict()
    assert min(d["fwd_ns"]) > 0 and min(d["bwd_ns"]) > 0
    assert 2000 < d["d2h_bytes_per_us"] < 400000 and 2000 < d["h2d_bytes_per_us"] < 400000   # some host link
    assert 0 < d["d2h_duplex_bytes_per_us"] <= d["d2h_bytes_per_us"] * 11 // 10
    assert 0 < d["h2d_duplex_bytes_per_us"] <= d["h2d_bytes_per_us"] * 11 // 10
    # the model of the unoptimised step is the sum of its nodes (Section 4.1, Eq. 1) and explains the measured step
    t_keep = timed(run, keep, 0)
    base = B.plan_cost(run.bcfg, cm, keep)["step_ns"]
    assert base == cfg.n_layers * (sum(d["fwd_ns"]) + sum(d["bwd_ns"]))
    assert 0.5 < base / t_keep < 2.0, (base, t_keep)      # (measured: within 15 %)
    _, vkeep = B.plan_validate(run.bcfg, keep)
    _, vlean = B.plan_validate(run.bcfg, syn.plan_all_recompute(cfg))
    lo, hi = vlean["peak_bytes"], vkeep["peak_bytes"]
    rows = []
    for frac in (0.8, 0.5, 0.2):
        budget = int(lo + frac * (hi - lo))
        code, plan, rep = B.plan_generate(run.bcfg, cm, budget, flags=B.MEMOPT_VALIDATE, raise_on_error=False)
        assert B.STATUS[code] == "DP_OK", (frac, B.last_error())
        run.poison_outputs()
        stats = run.step(plan, budget, want_stats=True)
        assert stats["peak_bytes"] <= budget
        assert all(torch.equal(a, b) for a, b in zip(want_bits, run.raw_results())), f"budget fraction {frac}"
        t = timed(run, plan, budget)
        rows.append((frac, budget, rep["moo_ns"], rep["exact_step_ns"], t))
        # predicted (the model's clocks on the executor's arena) against measured
        assert 0.5 < rep["exact_step_ns"] / t < 2.0, rows     # (measured: within 10 %)
        assert rep["exact_step_ns"] >= rep["base_ns"]
    print(name, "keep-all model/measured ns", base, int(t_keep), "| frac, budget, model moo, predicted, measured:", rows)
    # a tighter budget never gives a cheaper plan in the model
    assert rows[0][2] <= rows[1][2] <= rows[2][2]
    run.close()
