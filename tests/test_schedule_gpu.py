"""dp_stage_forward / dp_stage_backward through the C ABI: a stage fed several micro-batches
in one-forward-one-backward order, against the CPU oracle's schedule executor, plus the
properties that hold at any size (bits independent of plan, of the number in flight and of
the entry point used).  Metric and bounds as for dp_stage_step: max|gpu-ref| / max|ref| per
tensor, 1e-4 (fp32 debug mode), 2e-2 (bf16)."""
import dataclasses

import numpy as np
import pytest
import torch

import synthetic as syn
from oracle import stage as O
from paper_2505_05856_amd import binding as B
from paper_2505_05856_amd.harness import ScheduleRunner, StageRunner

pytestmark = pytest.mark.gpu
BOUND = {"f32": 1e-4, "bf16": 2e-2}


def make(cfg, n, sigma=0.05):
    w = syn.make_weights(cfg, sigma=sigma)
    xs, dys = [], []
    for m in range(n):
        x, dy = syn.make_activations(cfg, seed_x=11 + 2 * m, seed_dy=12 + 2 * m)
        xs.append(x); dys.append(dy)
    return w, xs, dys


def oracle_schedule(cfg, w, xs, dys, order, dtype=np.float64):
    st = O.Stage(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, cfg.micro_batch, cfg.norm_style,
                 cfg.causal, cfg.gelu, cfg.ln_eps)
    return O.stage_schedule(st, w, xs, dys, order, dtype=dtype)


def compare(cfg, got, ref):
    bound = BOUND[cfg.dtype]
    ys, dxs, g = got
    worst = {}
    for m, (a, b) in enumerate(zip(ys, ref[0])):
        worst[f"Y{m}"] = O.max_rel_err(a, b)
    for m, (a, b) in enumerate(zip(dxs, ref[1])):
        worst[f"dX{m}"] = O.max_rel_err(a, b)
    for l in range(cfg.n_layers):
        for k in syn.WEIGHT_NAMES:
            worst[f"L{l}.{k}"] = O.max_rel_err(g[l][k], ref[2][l][k])
    bad = {k: v for k, v in worst.items() if not (v <= bound)}
    print("largest errors:", ", ".join(f"{k}={v:.2e}" for k, v in sorted(worst.items(), key=lambda kv: -kv[1])[:4]))
    assert not bad, f"over {bound}: {bad}"


SMALL = [
    syn.StageConfig(2, 64, 2, 128, 40, 3, "pre", True, "erf", "f32"),
    syn.StageConfig(2, 64, 2, 128, 40, 3, "post", False, "tanh", "f32"),
    syn.StageConfig(3, 128, 2, 256, 96, 2, "pre", True, "erf", "bf16"),
    syn.StageConfig(2, 256, 2, 520, 130, 2, "post", False, "erf", "bf16"),      # ragged extents
]


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: f"{c.norm_style}-{c.dtype}-H{c.hidden}-S{c.seq}")
def test_schedule_matches_oracle_for_every_plan_and_depth(cfg):
    n = 4
    w, xs, dys = make(cfg, n)
    ref = oracle_schedule(cfg, w, xs, dys, O.one_f_one_b(n, 2))
    run = ScheduleRunner(cfg, w, xs, dys)
    B.stage_set_debug(run.stage, 2)      # poison released arena blocks
    plans = [("keep", syn.plan_keep_all(cfg)), ("recompute", syn.plan_all_recompute(cfg)),
             ("swap", syn.plan_all_swap(cfg)), ("c4", syn.plan_swap_ffn_recompute_norm_gelu(cfg)),
             ("seeded", syn.plan_seeded(cfg, 3)),
             ("mixed", [syn.plan_keep_all(cfg), syn.plan_all_swap(cfg), syn.plan_all_recompute(cfg),
                        syn.plan_seeded(cfg, 5)])]
    bits = None
    for inflight in (1, 2, 3, 4):
        for name, plan in plans:
            run.poison_outputs()
            run.run(O.one_f_one_b(n, inflight), inflight, plan)
            if bits is None:
                compare(cfg, run.results(), ref)
                bits = run.raw_results()
            else:
                assert all(torch.equal(a, b) for a, b in zip(bits, run.raw_results())), (inflight, name)
    run.close()


def test_each_micro_batch_equals_the_fused_step():
    """y, dx of every micro-batch and the gradients of a non-accumulating backward are the bits
    dp_stage_step writes; accumulated gradients are the running sum rounded once per backward."""
    cfg = SMALL[2]
    n = 3
    w, xs, dys = make(cfg, n)
    plan = syn.plan_swap_ffn_recompute_norm_gelu(cfg)
    sched = ScheduleRunner(cfg, w, xs, dys)
    sched.poison_outputs()
    sched.run(O.one_f_one_b(n, 2), 2, plan)
    ys, dxs, gsum = sched.results()
    running = None
    for m in range(n):
        one = StageRunner(cfg, w, xs[m], dys[m])
        one.step(plan)
        torch.cuda.synchronize()
        assert torch.equal(one.y, sched.y[m]) and torch.equal(one.dx, sched.dx[m])
        # a lone forward/backward pair with flags = 0 on a fresh slot writes the same gradients
        alone = ScheduleRunner(cfg, w, [xs[m]], [dys[m]])
        alone.poison_outputs()
        alone.run([("F", 0), ("B", 0)], 1, plan)
        torch.cuda.synchronize()
        for l in range(cfg.n_layers):
            for k in B.WEIGHT_FIELDS:
                assert torch.equal(one.g[l][k], alone.g[l][k]), (m, l, k)
        # the running sum in the storage dtype, one rounding per micro-batch
        if running is None:
            running = [{k: v.clone() for k, v in layer.items()} for layer in one.g]
        else:
            for l in range(cfg.n_layers):
                for k in B.WEIGHT_FIELDS:
                    running[l][k] = (running[l][k].float() + one.g[l][k].float()).to(running[l][k].dtype)
        one.close(); alone.close()
    # the fused step rounds each micro-batch's gradient before the sum and the schedule does
    # not, so the two agree to a few roundings of the storage type, not to the bit
    for l in range(cfg.n_layers):
        for k in B.WEIGHT_FIELDS:
            a, b = sched.g[l][k].float(), running[l][k].float()
            assert (a - b).abs().max().item() <= 2.0 ** -6 * b.abs().max().item(), (l, k)
    sched.close()


def test_budget_counts_every_micro_batch_in_flight():
    cfg = SMALL[2]
    w, xs, dys = make(cfg, 2)
    run = ScheduleRunner(cfg, w, xs, dys)
    plan = syn.plan_keep_all(cfg)
    _, rep = B.plan_validate(run.bcfg, plan)
    peak = rep["peak_bytes"]
    with pytest.raises(B.DpError) as e:
        run.forward(0, 2, plan, budget_bytes=2 * peak - 1)
    assert e.value.status == "DP_E_BUDGET"
    run.poison_outputs()
    run.run(O.one_f_one_b(2, 2), 2, plan, budget_bytes=2 * peak)
    ref = oracle_schedule(cfg, w, xs, dys, O.one_f_one_b(2, 2))
    compare(cfg, run.results(), ref)
    run.close()


def test_slot_misuse_is_an_error_and_leaves_the_handle_usable():
    cfg = SMALL[0]
    w, xs, dys = make(cfg, 2)
    run = ScheduleRunner(cfg, w, xs, dys)
    plan = syn.plan_keep_all(cfg)
    st = run.stage
    with pytest.raises(B.DpError) as e:
        B.stage_forward(st, 2, 2, run.x[0], plan, 0, run.y[0])            # slot not below inflight
    assert e.value.status == "DP_E_INVAL"
    with pytest.raises(B.DpError):
        B.stage_forward(st, 0, 0, run.x[0], plan, 0, run.y[0])            # inflight 0
    with pytest.raises(B.DpError):
        B.stage_forward(st, 0, 65, run.x[0], plan, 0, run.y[0])           # above the maximum
    with pytest.raises(B.DpError):
        B.stage_backward(st, 0, run.dy[0], run.dx[0], run.g)              # nothing fed yet
    B.stage_forward(st, 0, 2, run.x[0], plan, 0, run.y[0])
    with pytest.raises(B.DpError):
        B.stage_forward(st, 0, 2, run.x[1], plan, 0, run.y[1])            # slot occupied
    with pytest.raises(B.DpError):
        B.stage_backward(st, 0, run.dy[0], run.dx[0], run.g, flags=2)     # unknown flag; slot stays occupied
    with pytest.raises(B.DpError):
        B.stage_forward(st, 1, 2, run.x[1], plan[:-1], 0, run.y[1])       # the validator's errors come through
    B.stage_forward(st, 1, 2, run.x[1], plan, 0, run.y[1])
    B.stage_backward(st, 0, run.dy[0], run.dx[0], run.g)
    B.stage_backward(st, 1, run.dy[1], run.dx[1], run.g, flags=B.GRAD_ACCUMULATE)
    with pytest.raises(B.DpError):
        B.stage_backward(st, 1, run.dy[1], run.dx[1], run.g)              # already consumed
    ref = oracle_schedule(cfg, w, xs, dys, O.one_f_one_b(2, 2))
    compare(cfg, run.results(), ref)
    run.close()


def test_c2_full_size_schedule():
    """C2 at full size, four micro-batches, two in flight, under the swap+recompute plan and a
    budget of exactly two peaks: parity with the fp32 oracle and bits independent of the plan."""
    cfg = syn.CONFIGS["C2"]
    n = 4
    w, xs, dys = make(cfg, n, sigma=0.02)
    run = ScheduleRunner(cfg, w, xs, dys)
    plan = syn.plan_swap_ffn_recompute_norm_gelu(cfg)
    _, rep = B.plan_validate(run.bcfg, plan)
    run.poison_outputs()
    run.run(O.one_f_one_b(n, 2), 2, plan, budget_bytes=2 * rep["peak_bytes"])
    got = run.results()
    bits = run.raw_results()
    ref = oracle_schedule(cfg, w, xs, dys, O.one_f_one_b(n, 2), dtype=np.float32)
    compare(cfg, got, ref)
    run.poison_outputs()
    run.run(O.one_f_one_b(n, 3), 3, syn.plan_keep_all(cfg))
    assert all(torch.equal(a, b) for a, b in zip(bits, run.raw_results()))
    run.close()


# ---------------------------------------------------------------- parameter versions
def test_micro_batches_keep_the_parameter_version_of_their_forward():
    """An update after every backward, three micro-batches in flight: every micro-batch's y, dx
    and gradients are those of the version its forward saw (oracle), to the bit those of a fresh
    stage built from that version; the library holds exactly `inflight` versions at steady state."""
    cfg = SMALL[2]
    n, inflight = 6, 3
    _, xs, dys = make(cfg, n)
    versions = [syn.make_weights(cfg, seed=20 + v, sigma=0.05) for v in range(n + 1)]
    st = O.Stage(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, cfg.micro_batch, cfg.norm_style,
                 cfg.causal, cfg.gelu, cfg.ln_eps)
    order, v = [("W", 0)], 0
    for kind, m in O.one_f_one_b(n, inflight):
        order.append((kind, m))
        if kind == "B":
            v += 1
            order.append(("W", v))
    ref_y, ref_dx, ref_g, used, most = O.stage_schedule_async(st, versions, xs, dys, order)
    assert most == inflight

    from paper_2505_05856_amd.harness import upload
    run = ScheduleRunner(cfg, versions[0], xs, dys)
    plan = syn.plan_swap_ffn_recompute_norm_gelu(cfg)
    dev_versions = [[{k: upload(a, cfg) for k, a in layer.items()} for layer in ver] for ver in versions]
    grads_of = {}
    alive = []
    for kind, m in order:
        if kind == "W":
            B.stage_set_weights(run.stage, dev_versions[m])
        elif kind == "F":
            run.forward(m, inflight, plan)
        else:
            run.backward(m, accumulate=False)
            torch.cuda.synchronize()
            grads_of[m] = [{k: t.clone() for k, t in layer.items()} for layer in run.g]
        alive.append(B.stage_weight_versions(run.stage))
    assert max(alive) == inflight and alive[-1] == 1
    torch.cuda.synchronize()
    from paper_2505_05856_amd.harness import download
    for m in range(n):
        got = ([download(run.y[m])], [download(run.dx[m])], [{k: download(t) for k, t in layer.items()} for layer in grads_of[m]])
        compare(cfg, got, ([ref_y[m]], [ref_dx[m]], ref_g[m]))
        one = StageRunner(cfg, versions[used[m]], xs[m], dys[m])
        one.step(plan)
        torch.cuda.synchronize()
        assert torch.equal(one.y, run.y[m]) and torch.equal(one.dx, run.dx[m])
        assert all(torch.equal(one.g[l][k], grads_of[m][l][k]) for l in range(cfg.n_layers) for k in B.WEIGHT_FIELDS)
        one.close()
    run.close()


def test_set_weights_with_nothing_in_flight_updates_in_place():
    cfg = SMALL[0]
    w0, xs, dys = make(cfg, 1)
    w1 = syn.make_weights(cfg, seed=9, sigma=0.05)
    from paper_2505_05856_amd.harness import upload
    run = StageRunner(cfg, w0, xs[0], dys[0])
    run.step(syn.plan_keep_all(cfg))
    B.stage_set_weights(run.stage, [{k: upload(a, cfg) for k, a in layer.items()} for layer in w1])
    assert B.stage_weight_versions(run.stage) == 1
    run.poison_outputs()
    run.step(syn.plan_all_recompute(cfg))
    st = O.Stage(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, cfg.micro_batch, cfg.norm_style,
                 cfg.causal, cfg.gelu, cfg.ln_eps)
    y, dx, g = O.stage_step(st, w1, xs[0], dys[0])
    gy, gdx, gg = run.results()
    compare(cfg, ([gy], [gdx], gg), ([y], [dx], g))
    run.close()


def test_random_valid_event_orders_with_a_plan_per_micro_batch():
    """Any order in which every forward precedes its backward and at most `inflight` micro-batches are held:
    per-micro-batch results and the accumulated gradients equal the oracle's for that order, and y / dx do not
    depend on the order at all."""
    cfg = SMALL[3]
    n, inflight = 6, 3
    w, xs, dys = make(cfg, n)
    rng = np.random.default_rng(17)
    run = ScheduleRunner(cfg, w, xs, dys)
    B.stage_set_debug(run.stage, 2)
    first_bits = None
    for trial in range(4):
        order, fed, held, done = [], 0, [], 0
        while done < n:
            can_f = fed < n and len(held) < inflight
            if can_f and (not held or rng.random() < 0.5):
                order.append(("F", fed)); held.append(fed); fed += 1
            else:
                m = held.pop(int(rng.integers(len(held))))      # any held micro-batch, not only the oldest
                order.append(("B", m)); done += 1
        plans = [syn.plan_seeded(cfg, 50 * trial + m) for m in range(n)]
        ref = oracle_schedule(cfg, w, xs, dys, order)
        assert ref[3] <= inflight
        run.poison_outputs()
        run.run(order, inflight, plans)
        compare(cfg, run.results(), ref)
        bits = run.raw_results()[:2 * n]                          # y and dx of every micro-batch
        if first_bits is None:
            first_bits = bits
        assert all(torch.equal(a, b) for a, b in zip(first_bits, bits)), trial
    run.close()
