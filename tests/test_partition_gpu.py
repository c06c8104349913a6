"""dp_partition in front of the path, on the device: node times and link speed measured here,
a chain of BERT-Large-shaped layers cut into three stages under a budget that equal layer
counts cannot meet, then every stage of the result executed with its in-flight count under
that budget: it must run, give the bits of the all-KEEP plan, and take about the time the
search predicted."""
import dataclasses

import pytest
import torch

import synthetic as syn
from oracle import stage as O
from paper_2505_05856_amd import binding as B
from paper_2505_05856_amd.harness import ScheduleRunner, StageRunner, steady_state_ms, to_binding_config

pytestmark = pytest.mark.gpu


def test_partitioned_chain_runs_within_budget_and_near_prediction():
    layer = dataclasses.replace(syn.CONFIGS["C2"], n_layers=2)
    n, ell = 12, 3
    w = syn.make_weights(layer)
    x, dy = syn.make_activations(layer)
    probe = StageRunner(layer, w, x, dy)
    cm = B.stage_measure_cost_model(probe.stage, probe.x, probe.dy, probe.y, probe.dx, probe.g, steps=3)
    probe.close()
    one = dataclasses.replace(layer, n_layers=1)
    _, r1 = B.plan_validate(to_binding_config(one), syn.plan_keep_all(one))
    fl = r1["weight_bytes"] + r1["grad_bytes"]
    fs = r1["fixed_bytes"] - fl
    chain = to_binding_config(dataclasses.replace(layer, n_layers=n))
    _, loose = B.partition(chain, cm, ell, 0, fl, fs, flags=B.MEMOPT_VALIDATE)
    assert loose["cuts"] == [4, 8]
    need = max(s["peak_bytes"] * s["inflight"] for s in loose["stages"])
    budget = need * 55 // 100
    # equal layer counts: the first stage does not fit even with its own best plan
    first = to_binding_config(dataclasses.replace(layer, n_layers=4))
    code, _, _ = B.plan_generate(first, cm, budget, inflight=3, flags=B.MEMOPT_VALIDATE, raise_on_error=False)
    _, part = B.partition(chain, cm, ell, budget, fl, fs, flags=B.MEMOPT_VALIDATE)
    print("cuts", part["cuts"], "predicted ms", part["time_ns"] / 1e6, "equal layers fit:", code == 0,
          "memopt runs", part["n_memopt"], "positions", part["n_positions"])
    assert part["feasible"] and part["any_memopt"]
    assert part["cuts"] != loose["cuts"] or code == 0
    for s in part["stages"]:
        cfg = dataclasses.replace(layer, n_layers=s["n_layers"])
        k = s["inflight"]
        ws = syn.make_weights(cfg)
        xs, dys = [], []
        for m in range(k + 1):
            a, b = syn.make_activations(cfg, seed_x=31 + 2 * m, seed_dy=32 + 2 * m)
            xs.append(a); dys.append(b)
        run = ScheduleRunner(cfg, ws, xs, dys)
        order = O.one_f_one_b(k + 1, k)
        run.poison_outputs()
        run.run(order, k, s["plan"], budget_bytes=budget)          # validates inflight * peak <= budget
        bits = run.raw_results()
        run.poison_outputs()
        run.run(order, k, syn.plan_keep_all(cfg))
        assert all(torch.equal(p, q) for p, q in zip(bits, run.raw_results())), s["first_layer"]
        run.close()
        timed = StageRunner(cfg, ws, xs[0], dys[0])
        ms = steady_state_ms(timed, s["plan"], k, budget, 2, 6)
        timed.close()
        print(f"stage at layer {s['first_layer']}: {s['n_layers']} layers, {k} in flight, "
              f"predicted {s['time_ns'] / 1e6:.2f} ms, measured {ms:.2f} ms, memopt {s['memopt']}")
        assert 0.4 < ms / (s["time_ns"] / 1e6) < 2.5      # a gross disagreement only; the figures are printed above
