"""The planners on decoder stages (thirteen nodes and nineteen saved tensors a layer) against the
oracle: plan cost on seeded plans, generated plans, and the partition of a chain of decoder
layers -- all integers, so everything agrees exactly.  Host-only."""
import numpy as np
import pytest

import synthetic as syn
from oracle import memopt as M
from oracle import partition as P
from paper_2505_05856_amd import binding as B
from paper_2505_05856_amd.harness import to_binding_config

DEC = [syn.StageConfig(2, 64, 4, 256, 16, 2, "pre", True, "erf", "bf16", mem_seq=24),
       syn.StageConfig(3, 64, 2, 128, 32, 1, "pre", True, "erf", "bf16", mem_seq=5),
       syn.StageConfig(1, 128, 4, 512, 16, 2, "pre", False, "tanh", "f32", mem_seq=100)]


def both_sides(cfg):
    sh = M.StageShape(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, cfg.micro_batch, "dec",
                      2 if cfg.dtype == "bf16" else 4, cfg.mem_seq)
    return sh, to_binding_config(cfg)


def seeded_cost_model(seed, scale_ns, link):
    z = syn.splitmix64(seed, np.arange(26, dtype=np.uint64))
    t = [int(v % np.uint64(scale_ns)) + scale_ns // 10 for v in z]
    duplex = (max(1, link[0] * 3 // 4), max(1, link[1] * 4 // 5))
    return (M.CostModel(t[:13], t[13:], link[0], link[1], *duplex),
            B.make_cost_model(t[:13], t[13:], link[0], link[1], *duplex))


def test_the_oracles_decoder_tables_against_a_hand_count():
    """Keep-all: the step is the sum of all node times; the peak is every saved tensor of every layer but the
    stage input, plus the stage output's predecessor chain -- counted here from the shapes alone."""
    cfg = DEC[0]
    sh, _ = both_sides(cfg)
    ocm, _ = seeded_cost_model(3, 1000, (10**6, 10**6))
    r = M.plan_cost(sh, ocm, [M.KEEP] * (cfg.n_layers * sh.n_slots))
    assert sh.n_slots == 19 and r["step_ns"] == cfg.n_layers * (sum(ocm.fwd) + sum(ocm.bwd))
    T, Tm, H, F, e = cfg.tokens, cfg.mem_tokens, cfg.hidden, cfg.ffn, 2
    per_layer = (T * H * e * 9 + T * 3 * H * e + 2 * T * F * e + Tm * 2 * H * e + 3 * T * 8
                 + 2 * cfg.micro_batch * cfg.n_heads * cfg.seq * 4)
    # X_IN of layer 0 and the stage output are the caller's; layer 1's X_IN is layer 0's output
    assert r["peak_bytes"] == cfg.n_layers * per_layer - T * H * e
    # recomputing every KV_C costs one key/value projection a layer and takes all of them out of the peak (the
    # end of forward): when the top layer's comes back in backward, that layer's feed-forward tensors, which
    # are larger, have already been released
    p = [M.KEEP] * (cfg.n_layers * sh.n_slots)
    for l in range(cfg.n_layers):
        p[l * sh.n_slots + M.SLOT["KV_C"]] = M.RECOMPUTE
    r2 = M.plan_cost(sh, ocm, p)
    assert r2["step_ns"] == r["step_ns"] + cfg.n_layers * ocm.fwd[6] and r2["replayed"] == cfg.n_layers
    assert 2 * T * F * e > Tm * 2 * H * e
    assert r2["peak_bytes"] == r["peak_bytes"] - cfg.n_layers * Tm * 2 * H * e


@pytest.mark.parametrize("ci", range(len(DEC)))
def test_plan_cost_matches_the_oracle_on_seeded_plans(ci):
    cfg = DEC[ci]
    sh, bc = both_sides(cfg)
    for k, link in enumerate([(1000, 1000), (50, 80), (10**9, 10**9), (7, 3)]):
        ocm, cm = seeded_cost_model(100 + 10 * ci + k, 5000, link)
        plans = [syn.plan_seeded(cfg, 1000 * ci + seed) for seed in range(8)]
        plans += [syn.plan_keep_all(cfg), syn.plan_all_recompute(cfg), syn.plan_all_swap(cfg)]
        for i, plan in enumerate(plans):
            want = M.plan_cost(sh, ocm, list(plan), fixed_bytes=12345)
            got = B.plan_cost(bc, cm, plan, fixed_bytes=12345)
            assert got["step_ns"] == want["step_ns"], (ci, link, i)
            assert got["peak_bytes"] == want["peak_bytes"]
            assert (got["d2h_bytes"], got["h2d_bytes"], got["n_replayed_ops"]) == \
                   (want["d2h_bytes"], want["h2d_bytes"], want["replayed"])


@pytest.mark.parametrize("ci", range(len(DEC)))
def test_generated_plans_match_the_oracle(ci):
    cfg = DEC[ci]
    sh, bc = both_sides(cfg)
    for k, link in enumerate([(4000, 4000), (300, 500), (20, 20)]):
        ocm, cm = seeded_cost_model(7 + 31 * ci + k, 20000, link)
        keep_peak = M.plan_cost(sh, ocm, list(syn.plan_keep_all(cfg)), fixed_bytes=4096)["peak_bytes"]
        for frac in (100, 70, 40, 20, 5):
            for inflight in (1, 2):
                budget = keep_peak * frac // 100 * inflight
                want_plan, want = M.memopt(sh, ocm, budget, inflight, fixed_bytes=4096)
                code, got_plan, got = B.plan_generate(bc, cm, budget, inflight, fixed_bytes=4096, raise_on_error=False)
                assert list(got_plan) == want_plan, (ci, link, frac, inflight)
                assert B.STATUS[code] == ("DP_OK" if want["feasible"] else "DP_E_BUDGET")
                assert (got["base_ns"], got["moo_ns"], got["peak_bytes"]) == \
                       (want["base_ns"], want["moo_ns"], want["peak_bytes"])
                assert (got["n_free_swaps"], got["n_paid_swaps"], got["n_recomputed"]) == \
                       (want["free_swaps"], want["paid_swaps"], want["recomputed"])


def test_partition_of_a_decoder_chain_matches_the_oracle():
    layer = syn.StageConfig(1, 64, 4, 256, 16, 2, "pre", True, "erf", "bf16", mem_seq=24)
    args = (layer.hidden, layer.n_heads, layer.ffn, layer.seq, layer.micro_batch, "dec", 2, layer.mem_seq)
    ocm, cm = seeded_cost_model(77, 20000, (300, 300))
    n, fpl, fps = 6, 50_000, 20_000
    chain = P.Chain(args, ocm, n, fpl, fps)
    import dataclasses
    bc = to_binding_config(dataclasses.replace(layer, n_layers=n))
    keep_all = n * chain.mem_of(0) + fps
    for ell, frac in ((2, 0), (2, 30), (3, 40), (3, 26)):
        if True:
            budget = keep_all * frac // 100
            want = P.partition(chain, ell, budget)
            code, got = B.partition(bc, cm, ell, budget, fpl, fps, raise_on_error=False)
            assert got["feasible"] == want["feasible"], (ell, frac)
            if not want["feasible"]:
                continue
            assert got["cuts"] == want["cuts"] and got["time_ns"] == want["time_ns"], (ell, frac)
            for gs, ws in zip(got["stages"], want["stages"]):
                assert list(gs["plan"]) == ws["plan"] and gs["peak_bytes"] == ws["peak_bytes"]


def test_the_thread_count_does_not_change_a_plan():
    """The generator plays its trial plans on several host threads and reads them back in order: one thread or
    many, the plan and its figures are the same (a fresh process each, the count is read from the environment)."""
    import json
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = (
        "import json, sys, numpy as np\n"
        f"sys.path.insert(0, {root!r})\n"
        "import synthetic as syn\n"
        "from paper_2505_05856_amd import binding as B\n"
        "from paper_2505_05856_amd.harness import to_binding_config\n"
        "cfg = syn.StageConfig(3, 64, 2, 128, 32, 2, 'pre', True, 'erf', 'bf16', mem_seq=20)\n"
        "bc = to_binding_config(cfg)\n"
        "cm = B.make_cost_model([900 + 37 * i for i in range(13)], [1700 + 53 * i for i in range(13)], 40, 60)\n"
        "_, keep = B.plan_validate(bc, syn.plan_keep_all(cfg))\n"
        "out = []\n"
        "for frac in (80, 60, 45):\n"
        "    code, plan, rep = B.plan_generate(bc, cm, keep['peak_bytes'] * frac // 100, 2, flags=B.MEMOPT_VALIDATE, raise_on_error=False)\n"
        "    out.append([code, [int(v) for v in plan], rep['moo_ns'], rep['peak_bytes'], rep['exact_step_ns']])\n"
        "print(json.dumps(out))\n")
    results = []
    for threads in ("1", "5"):
        env = dict(os.environ, DPSTAGE_PLANNER_THREADS=threads)
        p = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=300)
        assert p.returncode == 0, p.stderr[-2000:]
        results.append(json.loads(p.stdout.strip().splitlines()[-1]))
    assert results[0] == results[1]
    assert any(sum(r[1]) > 0 for r in results[0])       # (budgets that do need a plan)
