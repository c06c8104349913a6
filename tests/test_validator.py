"""Host-only tests: the library loads, exports what the header declares, and the
plan validator's memory walk obeys the accounting rule of Algorithm 2 (add what
is allocated, take the running maximum, subtract what is released) and the
feasibility test of Algorithm 1 (inflight x peak against the capacity)."""
import ctypes
import os
import re

import numpy as np
import pytest

import synthetic as syn
from paper_2505_05856_amd import binding as B
from paper_2505_05856_amd.harness import to_binding_config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "dpstage.h")).read()
    names = sorted(set(re.findall(r"\b(dp_[a-z_]+)\s*\(", hdr)))
    assert "dp_stage_step" in names and "dp_plan_validate" in names and len(names) >= 17
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n


def small(style="pre", L=2):
    return syn.StageConfig(L, 64, 2, 128, 16, 2, style, style == "pre", "erf", "bf16")


def test_argument_errors():
    cfg = small()
    bc = to_binding_config(cfg)
    n = syn.plan_len(cfg)
    assert B.plan_len(bc) == n == cfg.n_layers * 12
    code, _ = B.plan_validate(bc, None, raise_on_error=False)
    assert B.STATUS[code] == "DP_E_INVAL"
    code, _ = B.plan_validate(bc, np.zeros(n - 1, np.uint8), raise_on_error=False)
    assert B.STATUS[code] == "DP_E_INVAL" and "plan_len" in B.last_error()
    p = syn.plan_keep_all(cfg); p[5] = 3
    code, rep = B.plan_validate(bc, p, raise_on_error=False)
    assert B.STATUS[code] == "DP_E_INVAL" and rep["first_bad_slot"] == 5
    p = syn.plan_keep_all(cfg); p[syn.SLOT["X_IN"]] = syn.RECOMPUTE
    code, rep = B.plan_validate(bc, p, raise_on_error=False)
    assert B.STATUS[code] == "DP_E_PLAN" and (rep["first_bad_layer"], rep["first_bad_slot"]) == (0, 0)
    code, _ = B.plan_validate(bc, syn.plan_keep_all(cfg), inflight=0, raise_on_error=False)
    assert B.STATUS[code] == "DP_E_INVAL"
    bad = B.make_config(1, 60, 4, 128, 16, 2)   # head_dim 15
    assert B.plan_len(bad) == 0
    code, _ = B.plan_validate(bad, np.zeros(12, np.uint8), raise_on_error=False)
    assert B.STATUS[code] == "DP_E_UNSUPPORTED"
    bad = B.make_config(1, 64, 3, 128, 16, 2)   # hidden not a multiple of heads
    code, _ = B.plan_validate(bad, np.zeros(12, np.uint8), raise_on_error=False)
    assert B.STATUS[code] == "DP_E_INVAL"


def r256(n):
    return (n + 255) // 256 * 256


@pytest.mark.parametrize("style", ["pre", "post"])
def test_keep_all_peak_by_hand(style):
    """Keep-all: every slot of every layer is live at the forward/backward
    turnaround; on top of that sits the largest transient set of the last
    layer's backward."""
    cfg = small(style, L=3)
    bc = to_binding_config(cfg)
    _, rep = B.plan_validate(bc, syn.plan_keep_all(cfg))
    T, H, F, e = cfg.tokens, cfg.hidden, cfg.ffn, 2
    th, tf, st, lse = r256(T * H * e), r256(T * F * e), r256(T * 8), r256(cfg.micro_batch * cfg.n_heads * cfg.seq * 4)
    per_layer = 4 * th + r256(3 * T * H * e) + 2 * tf + 2 * st + lse     # LN1_OUT,ATTN_OUT,RES1,(LN2_OUT|RES2); QKV; FC1,GELU
    slots = cfg.n_layers * per_layer + (cfg.n_layers - 1) * th          # + X_IN of layers 1..L-1
    assert rep["kept_act_bytes"] == cfg.n_layers * (per_layer - 4 * th - r256(3 * T * H * e) - 2 * tf - 2 * st - lse) + \
        cfg.n_layers * (4 * T * H * e + 3 * T * H * e + 2 * T * F * e + 2 * T * 8 + cfg.micro_batch * cfg.n_heads * cfg.seq * 4) + \
        (cfg.n_layers - 1) * T * H * e
    # the walk's peak is at least all slots plus the first backward transient (dG or dR2)
    assert rep["live_peak_bytes"] - rep["fixed_bytes"] >= slots + min(th, tf)
    assert rep["live_peak_bytes"] - rep["fixed_bytes"] <= slots + 2 * tf + 2 * th + r256(T // 8 * 2 * max(F, 3 * H) * 4)
    assert rep["arena_peak_bytes"] >= rep["live_peak_bytes"] - rep["fixed_bytes"]
    assert rep["peak_bytes"] == rep["fixed_bytes"] + rep["arena_peak_bytes"]
    # fixed part: weights (as given + transposed matrices), gradients, x/dy/y/dx
    mats = 3 * H * H + H * H + 2 * H * F
    vecs = 9 * H + F
    assert rep["weight_bytes"] == cfg.n_layers * (2 * mats + vecs) * e
    assert rep["grad_bytes"] == cfg.n_layers * (mats + vecs) * e
    assert rep["fixed_bytes"] == rep["weight_bytes"] + rep["grad_bytes"] + 4 * T * H * e
    assert rep["n_replayed_ops"] == 0 and rep["swap_out_bytes"] == 0 and rep["replay_flops"] == 0
    assert abs(rep["step_flops"] - cfg.model_flops()) < 1e-6 * cfg.model_flops()


@pytest.mark.parametrize("style", ["pre", "post"])
def test_plans_reduce_peak_and_account_traffic(style):
    cfg = small(style, L=4)
    bc = to_binding_config(cfg)
    _, keep = B.plan_validate(bc, syn.plan_keep_all(cfg))
    _, rec = B.plan_validate(bc, syn.plan_all_recompute(cfg))
    _, swp = B.plan_validate(bc, syn.plan_all_swap(cfg))
    assert rec["live_peak_bytes"] < keep["live_peak_bytes"] and swp["live_peak_bytes"] < keep["live_peak_bytes"]
    assert rec["peak_bytes"] < keep["peak_bytes"] and swp["peak_bytes"] < keep["peak_bytes"]
    # all-recompute replays each layer's forward: all but the last op in pre-LN (its
    # output is the kept next-layer input); post-LN also reruns LN2 for its statistics
    assert rec["n_replayed_ops"] == cfg.n_layers * (7 if style == "pre" else 8)
    fwd = cfg.model_flops() / 3
    last_gemm = 2 * cfg.tokens * cfg.hidden * cfg.ffn * cfg.n_layers      # FC2 (pre) is never replayed
    expect = fwd - last_gemm if style == "pre" else fwd
    assert abs(rec["replay_flops"] - expect) < 1e-6 * fwd
    # all-swap: every stored slot goes out once and comes back once
    assert swp["swap_out_bytes"] == swp["swap_in_bytes"] == keep["kept_act_bytes"]
    assert swp["host_pinned_bytes"] >= swp["swap_out_bytes"] and swp["n_replayed_ops"] == 0
    assert swp["n_swapped_slots"] == cfg.n_layers * 11 - 1


def test_single_slot_monotonicity():
    """Turning one more slot from KEEP to RECOMPUTE or SWAP never raises the walk's peak."""
    cfg = small("pre", L=3)
    bc = to_binding_config(cfg)
    base = syn.plan_keep_all(cfg)
    _, rb = B.plan_validate(bc, base)
    for i in range(len(base)):
        l, s = divmod(i, 12)
        if s in cfg.alias_slots() or (l == 0 and s == 0):
            continue
        for a in (syn.RECOMPUTE, syn.SWAP):
            p = base.copy(); p[i] = a
            _, r = B.plan_validate(bc, p)
            assert r["live_peak_bytes"] <= rb["live_peak_bytes"], (l, s, a)


def test_budget_predicate():
    cfg = small("pre", L=2)
    bc = to_binding_config(cfg)
    p = syn.plan_keep_all(cfg)
    _, rep = B.plan_validate(bc, p)
    peak = rep["peak_bytes"]
    assert B.plan_validate(bc, p, budget_bytes=peak)[0] == 0            # equal budget must run
    code, rep2 = B.plan_validate(bc, p, budget_bytes=peak - 1, raise_on_error=False)
    assert B.STATUS[code] == "DP_E_BUDGET" and rep2["peak_bytes"] == peak
    assert B.plan_validate(bc, p, budget_bytes=4 * peak, inflight=4)[0] == 0
    code, _ = B.plan_validate(bc, p, budget_bytes=4 * peak - 1, inflight=4, raise_on_error=False)
    assert B.STATUS[code] == "DP_E_BUDGET"
    # a plan that frees memory fits where keep-all does not
    _, rr = B.plan_validate(bc, syn.plan_all_recompute(cfg))
    assert B.plan_validate(bc, syn.plan_all_recompute(cfg), budget_bytes=rr["peak_bytes"])[0] == 0
    assert rr["peak_bytes"] < peak


def test_swap_policy_ladder_spends_exactly_the_headroom():
    """A swapping plan under budgets from generous down to its minimum: every budget at or above the minimum is
    feasible, the validated peak never exceeds the budget and never grows when the budget shrinks, the most
    generous policy (blocks held, copy-outs of the upper layers deferred to the end of the forward) needs no more
    than keeping everything, the traffic is the plan's whatever the policy, and half the minimum fails."""
    for cfg in (small("pre", L=4), small("post", L=3)):
        bc = to_binding_config(cfg)
        for plan in (syn.plan_all_swap(cfg), syn.plan_seeded(cfg, 7), syn.plan_seeded(cfg, 11)):
            _, tight = B.plan_validate(bc, plan)                       # no budget: the tightest policy
            _, keep = B.plan_validate(bc, syn.plan_keep_all(cfg))
            _, roomy = B.plan_validate(bc, plan, budget_bytes=1 << 40)
            lo, hi = tight["peak_bytes"], roomy["peak_bytes"]
            assert lo <= hi <= keep["peak_bytes"] + 4096 * 64          # (alignment slack of the arena)
            assert roomy["swap_out_bytes"] == tight["swap_out_bytes"] and roomy["swap_in_bytes"] == tight["swap_in_bytes"]
            last = hi
            for k in range(9):
                budget = hi - (hi - lo) * k // 8
                code, rep = B.plan_validate(bc, plan, budget_bytes=budget, raise_on_error=False)
                assert code == 0, (k, budget, B.last_error())
                assert rep["peak_bytes"] <= budget and rep["peak_bytes"] <= last
                assert rep["swap_out_bytes"] == tight["swap_out_bytes"]
                last = rep["peak_bytes"]
            # (first-fit fragmentation can make another policy a few blocks smaller than the tightest one)
            assert lo - 64 * 4096 <= last <= lo
            code, _ = B.plan_validate(bc, plan, budget_bytes=lo // 2, raise_on_error=False)
            assert B.STATUS[code] == "DP_E_BUDGET"


def test_ignored_plan_bytes_and_random_plans():
    cfg = small("post", L=3)
    bc = to_binding_config(cfg)
    a = syn.plan_keep_all(cfg)
    b = a.copy()
    b.reshape(3, 12)[:, syn.SLOT["LN2_OUT"]] = syn.SWAP     # no storage in post-LN
    b[syn.SLOT["X_IN"]] = syn.SWAP                          # caller memory
    assert B.plan_validate(bc, a)[1] == B.plan_validate(bc, b)[1]
    for seed in range(200):
        for c in (cfg, small("pre", L=3)):
            code, rep = B.plan_validate(to_binding_config(c), syn.plan_seeded(c, seed))
            assert code == 0 and rep["arena_peak_bytes"] >= rep["live_peak_bytes"] - rep["fixed_bytes"] > 0
            assert rep["swap_in_bytes"] <= rep["swap_out_bytes"]


def test_full_size_configs_fit_their_budgets():
    for name, cfg in syn.CONFIGS.items():
        bc = to_binding_config(cfg)
        for pname, mk in syn.PLANS[name]:
            code, rep = B.plan_validate(bc, mk(cfg), budget_bytes=syn.BUDGETS.get(name, 0))
            assert code == 0, (name, pname, B.last_error())
            assert rep["peak_bytes"] < 288 * 10**9


def test_a_shape_the_matrix_core_kernels_do_not_take_is_reported_up_front():
    """The vector-ALU kernels behind an unsupported shape are 20-50 times slower: the memory report says how many
    launches of a step take them (and dp_step_stats repeats it), so a caller sees the cliff before running."""
    for name in ("C2", "C3", "C4", "C5"):
        cfg = syn.CONFIGS[name]
        _, rep = B.plan_validate(to_binding_config(cfg), syn.PLANS[name][0][1](cfg), budget_bytes=syn.BUDGETS.get(name, 0))
        assert rep["n_fallback_launches"] == 0, name
    # head dimension 96: attention forward and backward of each of the 2 layers fall back, the GEMMs do not
    odd = syn.StageConfig(2, 192, 2, 384, 64, 2, "pre", True, "erf", "bf16")
    _, rep = B.plan_validate(to_binding_config(odd), syn.plan_keep_all(odd))
    assert rep["n_fallback_launches"] == 4
    # a replayed attention counts again
    _, rep = B.plan_validate(to_binding_config(odd), syn.plan_all_recompute(odd))
    assert rep["n_fallback_launches"] == 6
    # fp32 debug mode runs on the vector ALUs by definition: nothing "fell back"
    f32 = syn.StageConfig(2, 192, 2, 384, 64, 2, "pre", True, "erf", "f32")
    assert B.plan_validate(to_binding_config(f32), syn.plan_keep_all(f32))[1]["n_fallback_launches"] == 0


# ---------------------------------------------------------------- decoder stages (cross-attention block)
def _dec(**kw):
    base = dict(n_layers=2, hidden=128, n_heads=2, ffn=256, seq=64, micro_batch=2, norm_style="pre", causal=True,
                dtype="bf16", mem_seq=40)
    base.update(kw)
    return syn.StageConfig(**base)


def test_decoder_stage_plans_and_memory():
    cfg = _dec()
    bc = to_binding_config(cfg)
    assert B.plan_len(bc) == cfg.n_layers * B.SLOTS_PER_LAYER_CROSS == syn.plan_len(cfg)
    _, keep = B.plan_validate(bc, syn.plan_keep_all(cfg))
    _, rec = B.plan_validate(bc, syn.plan_all_recompute(cfg))
    assert keep["step_flops"] == cfg.model_flops() and keep["n_replayed_ops"] == 0
    assert rec["arena_peak_bytes"] < keep["arena_peak_bytes"] and rec["n_replayed_ops"] == 12 * cfg.n_layers
    # what keep-all holds: the plain layer's saved tensors plus the block's seven
    T, Tm, H, e = cfg.tokens, cfg.mem_tokens, cfg.hidden, 2
    block = 4 * T * H * e + Tm * 2 * H * e + T * 2 * 4 + cfg.micro_batch * cfg.n_heads * cfg.seq * 4
    _, plain = B.plan_validate(to_binding_config(syn.small_like(cfg, mem_seq=0)), syn.plan_keep_all(syn.small_like(cfg, mem_seq=0)))
    assert keep["kept_act_bytes"] == plain["kept_act_bytes"] + cfg.n_layers * block
    # recomputing KV_C alone costs one projection of the memory a layer and frees its bytes
    _, kv = B.plan_validate(bc, syn.plan_from_slots(cfg, {"KV_C": syn.RECOMPUTE}))
    assert kv["n_replayed_ops"] == cfg.n_layers and kv["replay_flops"] == cfg.n_layers * 2.0 * Tm * H * 2 * H
    assert kv["kept_act_bytes"] == keep["kept_act_bytes"] - cfg.n_layers * Tm * 2 * H * e
    # the encoder memory and its gradient count as fixed memory
    assert keep["fixed_bytes"] - plain["fixed_bytes"] >= 2 * Tm * H * e


def test_decoder_stage_refusals():
    for bad in (_dec(norm_style="post"), _dec(mem_seq=-1)):
        with pytest.raises(B.DpError):
            B.plan_validate(to_binding_config(bad), syn.plan_keep_all(_dec()))
    cfg = _dec()
    with pytest.raises(B.DpError):      # a plain stage's plan length
        B.plan_validate(to_binding_config(cfg), np.zeros(cfg.n_layers * B.SLOTS_PER_LAYER, dtype=np.uint8))
    # the planners take a decoder stage with a thirteen-node cost model; without a budget nothing is changed
    cm = B.make_cost_model([1000] * 13, [2000] * 13, 50_000, 50_000)
    code, plan, rep = B.plan_generate(to_binding_config(cfg), cm, 0, 1)
    assert len(plan) == syn.plan_len(cfg) and not plan.any() and rep["base_ns"] == cfg.n_layers * 13 * 3000
