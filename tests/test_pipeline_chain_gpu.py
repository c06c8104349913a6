"""The pieces put together as the paper uses them (Sections 1, 4.2, 4.3): a chain of layers is cut into
stages by dp_partition under a device budget that forces memory optimisation on the early stages, every
stage gets its own handle and its own plan, and the stages run a one-forward-one-backward schedule over
several micro-batches, handing activations forward and gradients back -- all on one GPU, in an order that
respects the dependencies between stages.  The outputs, the input gradients and the gradients summed over
the micro-batches must be those of the oracle's unpartitioned chain, and stage x of l must never hold
more than l - x + 1 micro-batches."""
import dataclasses

import numpy as np
import pytest
import torch

import synthetic as syn
from oracle import stage as O
from paper_2505_05856_amd import binding as B
from paper_2505_05856_amd.harness import download, to_binding_config, upload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("ell,n_micro,frac", [(3, 5, 0.8), (2, 3, 0.6)])
def test_partitioned_chain_under_1f1b_matches_the_unpartitioned_oracle(ell, n_micro, frac):
    chain = syn.StageConfig(6, 128, 2, 256, 128, 4, "pre", True, "erf", "bf16")
    w = syn.make_weights(chain, sigma=0.05)
    xs, dys = [], []
    for m in range(n_micro):
        x, dy = syn.make_activations(chain, seed_x=100 + m, seed_dy=200 + m)
        xs.append(x); dys.append(dy)
    # the cut: node times of a plausible shape, a slow link, and a budget below what stage 1 needs to keep everything
    cm = B.make_cost_model([4000, 30000, 20000, 12000, 4000, 25000, 6000, 25000],
                           [50000, 8000, 50000, 6000, 24000, 45000, 55000, 6000], 3000, 3000)
    one = dataclasses.replace(chain, n_layers=1)
    _, r1 = B.plan_validate(to_binding_config(one), syn.plan_keep_all(one))
    fpl = r1["weight_bytes"] + r1["grad_bytes"]
    equal = dataclasses.replace(chain, n_layers=chain.n_layers // ell)
    _, req = B.plan_validate(to_binding_config(equal), syn.plan_keep_all(equal))
    budget = int(ell * req["peak_bytes"] * frac)      # of what equal layer counts would hold on stage 1
    _, part = B.partition(to_binding_config(chain), cm, ell, budget, fpl, r1["fixed_bytes"] - fpl, flags=B.MEMOPT_VALIDATE)
    assert part["feasible"] and part["any_memopt"]
    stages = part["stages"]
    assert sum(s["n_layers"] for s in stages) == chain.n_layers
    # one handle per stage
    handles, grads, cfgs = [], [], []
    for s in stages:
        a, n = s["first_layer"], s["n_layers"]
        c = dataclasses.replace(chain, n_layers=n)
        tw = [{k: upload(v, c) for k, v in layer.items()} for layer in w[a:a + n]]
        handles.append(B.stage_init(to_binding_config(c), tw, 0))
        grads.append([{k: torch.full_like(v, float("nan")) for k, v in layer.items()} for layer in tw])
        cfgs.append(c)
        assert s["inflight"] == ell - len(handles) + 1
    T, H = chain.tokens, chain.hidden
    dt = torch.bfloat16
    act = [[None] * n_micro for _ in range(ell + 1)]       # act[x][m]: input of stage x (act[ell]: the chain's output)
    gin = [[None] * n_micro for _ in range(ell + 1)]       # gin[x][m]: gradient of stage x's output ... gin[0]: dX
    for m in range(n_micro):
        act[0][m] = upload(xs[m], chain)
        gin[ell][m] = upload(dys[m], chain)
    # every stage follows its own one-forward-one-backward order; a global loop runs whatever is ready
    orders = [list(O.one_f_one_b(n_micro, ell - x)) for x in range(ell)]
    pos = [0] * ell
    slot_of = [dict() for _ in range(ell)]
    most = [0] * ell
    nb = [0] * ell
    while any(pos[x] < len(orders[x]) for x in range(ell)):
        progressed = False
        for x in range(ell):
            if pos[x] == len(orders[x]):
                continue
            kind, m = orders[x][pos[x]]
            k = ell - x
            if kind == "F":
                if act[x][m] is None:
                    continue
                slot = min(s for s in range(k) if s not in slot_of[x].values())
                y = torch.empty(T, H, dtype=dt, device="cuda:0")
                B.stage_forward(handles[x], slot, k, act[x][m], stages[x]["plan"], budget, y)
                act[x + 1][m] = y
                slot_of[x][m] = slot
                most[x] = max(most[x], len(slot_of[x]))
            else:
                if gin[x + 1][m] is None:
                    continue
                dx = torch.empty(T, H, dtype=dt, device="cuda:0")
                B.stage_backward(handles[x], slot_of[x].pop(m), gin[x + 1][m], dx, grads[x],
                                 B.GRAD_ACCUMULATE if nb[x] else 0)
                nb[x] += 1
                gin[x][m] = dx
            pos[x] += 1
            progressed = True
        assert progressed, "the schedule deadlocked"
    torch.cuda.synchronize()
    assert most == [min(ell - x, n_micro) for x in range(ell)]
    # the unpartitioned chain on the oracle
    st = O.Stage(chain.n_layers, chain.hidden, chain.n_heads, chain.ffn, chain.seq, chain.micro_batch, "pre", True, "erf",
                 chain.ln_eps)
    ys, dxs, total, _ = O.stage_schedule(st, w, xs, dys, O.one_f_one_b(n_micro, 1))
    worst = 0.0
    for m in range(n_micro):
        worst = max(worst, O.max_rel_err(download(act[ell][m]), ys[m]), O.max_rel_err(download(gin[0][m]), dxs[m]))
    for x, s in enumerate(stages):
        for i in range(s["n_layers"]):
            for name in syn.WEIGHT_NAMES:
                worst = max(worst, O.max_rel_err(download(grads[x][i][name]), total[s["first_layer"] + i][name]))
    print(f"cuts {part['cuts']}, worst max-rel-err {worst:.3e}")
    assert worst <= 2e-2
    for h in handles:
        h.close()
