"""Dropout on the device against the CPU oracle, through the C ABI: the mask bits exactly, the
operators and the stage step to the stage's bounds (max|gpu-ref| / max|ref| <= 1e-4 fp32,
2e-2 bf16), and the property the method needs: a plan does not change a single bit, i.e. a
recomputed tensor meets the mask of its first computation."""
import dataclasses
import warnings

import numpy as np
import pytest
import torch

import synthetic as syn
from oracle import dropout as D
from oracle import stage as O
from paper_2505_05856_amd import binding as B
from paper_2505_05856_amd.harness import ScheduleRunner, StageRunner
from test_ops_gpu import DEV, TOL, dev, host, rnd, ws_for
from test_stage_gpu import compare

pytestmark = pytest.mark.gpu
warnings.filterwarnings("ignore", message="overflow encountered")


def oracle_stage(cfg):
    return O.Stage(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, cfg.micro_batch, cfg.norm_style,
                   cfg.causal, cfg.gelu, cfg.ln_eps, p_attn=cfg.p_attn, p_hidden=cfg.p_hidden)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("T,H", [(1, 8), (37, 24), (200, 328), (1031, 1024)])
@pytest.mark.parametrize("p", [0.1, 0.5])
def test_hidden_mask_is_the_oracles_bit_for_bit(dt, T, H, p):
    seed, mb, layer = 0x1234_5678_9ABC_DEF0, 7 + (3 << 32), 5
    drop = B.Dropout(p, seed, mb, layer)
    ones = torch.ones(T, H, dtype=dt, device=DEV)
    for site in (B.SITE_PROJ, B.SITE_FC2):
        y = torch.empty_like(ones)
        B.op_dropout(ones, None, y, drop, site)
        keep = D.keep_hidden(seed, mb, layer, site, T, H, p)
        got = host(y)
        assert np.array_equal(got != 0, keep)
        assert np.allclose(got[keep], D.scale(p), rtol=TOL[dt])
    # with a residual, in place, against the oracle's arithmetic
    x, res = rnd((T, H), 61, dt), rnd((T, H), 62, dt)
    tx, tres = dev(x, dt), dev(res, dt)
    B.op_dropout(tx, tres, tx, drop, B.SITE_PROJ)
    keep = D.keep_hidden(seed, mb, layer, B.SITE_PROJ, T, H, p)
    ref = res.astype(np.float64) + x.astype(np.float64) * keep * D.scale(p)
    assert O.max_rel_err(host(tx), ref) < TOL[dt]
    assert np.array_equal(host(tx)[~keep], res.astype(np.float64)[~keep])     # dropped: the residual, untouched


def test_dropout_rate_zero_and_bad_arguments():
    x = dev(rnd((16, 16), 1, torch.float32), torch.float32)
    y = torch.empty_like(x)
    B.op_dropout(x, None, y, B.Dropout(0.0, 1, 2, 0), B.SITE_FC2)
    assert torch.equal(x, y)
    for bad in (B.Dropout(1.0, 1, 2, 0), B.Dropout(-0.1, 1, 2, 0), B.Dropout(0.1, 1, 2, -1)):
        with pytest.raises(B.DpError):
            B.op_dropout(x, None, y, bad, B.SITE_FC2)
    with pytest.raises(B.DpError):
        B.op_dropout(x, None, y, B.Dropout(0.1, 1, 2, 0), 0)          # site 0 is the attention's
    with pytest.raises(B.DpError):
        B.op_dropout(x.flatten()[:12], None, y.flatten()[:12], B.Dropout(0.1, 1, 2, 0), 1)


ATTN_SHAPES = [(1, 8, 1, 8), (2, 5, 2, 16), (2, 64, 2, 64), (1, 200, 3, 64), (2, 96, 2, 128), (1, 384, 2, 64),
               (1, 300, 1, 128)]


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Bn,S,nh,dh", ATTN_SHAPES)
def test_attention_with_dropout(dt, causal, Bn, S, nh, dh):
    H = nh * dh
    p, seed, mb, layer = 0.25, 99, 3, 2
    qkv = rnd((Bn * S, 3 * H), 51, dt)
    d_o = rnd((Bn * S, H), 52, dt)
    q64 = qkv.astype(np.float64)
    keep = lambda b: D.keep_attention(seed, mb, layer, b, nh, S, p)
    o_ref, lse_ref = O.attention_fwd(q64, Bn, S, nh, causal, keep, D.scale(p))
    dq_ref = O.attention_bwd(d_o.astype(np.float64), q64, Bn, S, nh, causal, keep, D.scale(p))
    plain, _ = O.attention_fwd(q64, Bn, S, nh, causal)
    tq, tdo = dev(qkv, dt), dev(d_o, dt)
    o = torch.empty(Bn * S, H, dtype=dt, device=DEV)
    lse = torch.empty(Bn, nh, S, dtype=torch.float32, device=DEV)
    drop = B.Dropout(p, seed, mb, layer)
    B.op_attention_dropout_fwd(tq, Bn, S, nh, dh, causal, o, lse, drop)
    tol = TOL[dt] * (2 if dt == torch.bfloat16 else 1)
    err = O.max_rel_err(host(o), o_ref)
    assert err < tol, err
    if S >= 64:
        assert O.max_rel_err(host(o), plain) > 20 * tol                 # the mask did something
    assert np.allclose(host(lse), lse_ref, atol=2e-5 if dt == torch.float32 else 2e-3)
    dqkv = torch.empty_like(tq)
    ws = ws_for(Bn * S, nh)
    B.op_attention_dropout_bwd(tq, o, lse, tdo, Bn, S, nh, dh, causal, dqkv, ws, drop)
    got = host(dqkv)
    for blk in range(3):
        e = O.max_rel_err(got[:, blk * H:(blk + 1) * H], dq_ref[:, blk * H:(blk + 1) * H])
        assert e < 2 * tol, (blk, e)
    # rate 0 through the dropout entry point is the plain operator, to the bit
    o0, o1 = torch.empty_like(o), torch.empty_like(o)
    B.op_attention_dropout_fwd(tq, Bn, S, nh, dh, causal, o0, None, B.Dropout(0.0, seed, mb, layer))
    B.op_attention_fwd(tq, Bn, S, nh, dh, causal, o1, None)
    assert torch.equal(o0, o1)


SMALL = [
    syn.StageConfig(2, 64, 2, 128, 40, 3, "pre", True, "erf", "f32", p_attn=0.2, p_hidden=0.1),
    syn.StageConfig(2, 64, 2, 128, 40, 3, "post", False, "tanh", "f32", p_attn=0.1, p_hidden=0.3),
    syn.StageConfig(3, 128, 2, 256, 96, 2, "pre", True, "erf", "bf16", p_attn=0.1, p_hidden=0.1),
    syn.StageConfig(3, 128, 2, 256, 96, 2, "post", False, "erf", "bf16", p_attn=0.1, p_hidden=0.1),
    syn.StageConfig(2, 256, 2, 520, 130, 2, "pre", True, "tanh", "bf16", p_attn=0.0, p_hidden=0.2),
    syn.StageConfig(2, 256, 2, 520, 130, 2, "post", True, "erf", "bf16", p_attn=0.3, p_hidden=0.0),
]


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: f"{c.norm_style}-{c.dtype}-H{c.hidden}-pa{c.p_attn}-ph{c.p_hidden}")
def test_stage_step_with_dropout_every_plan(cfg):
    w = syn.make_weights(cfg, sigma=0.05)
    x, dy = syn.make_activations(cfg)
    seed, mb = 0xABCDEF0123, 41
    st = oracle_stage(cfg)
    st.set_rng(seed, mb)
    ref = O.stage_step(st, w, x, dy)
    run = StageRunner(cfg, w, x, dy)
    B.stage_set_debug(run.stage, 2)      # poison released arena blocks
    plans = [syn.plan_keep_all(cfg), syn.plan_all_recompute(cfg), syn.plan_uniform(cfg, syn.RECOMPUTE),
             syn.plan_all_swap(cfg), syn.plan_swap_ffn_recompute_norm_gelu(cfg), syn.plan_seeded(cfg, 7)]
    bits = None
    for plan in plans:
        B.stage_set_rng(run.stage, seed, mb)
        run.poison_outputs()
        run.step(plan)
        if bits is None:
            compare(cfg, run.results(), ref)
            bits = run.raw_results()
        else:
            assert all(torch.equal(a, b) for a, b in zip(bits, run.raw_results()))
    # the counter advanced: the next step draws other masks; setting it back repeats the first
    run.step(plans[0])
    assert not torch.equal(bits[0], run.raw_results()[0])
    st.set_rng(seed, mb + 1)
    compare(cfg, run.results(), O.stage_step(st, w, x, dy))
    B.stage_set_rng(run.stage, seed, mb)
    run.step(plans[1])
    assert all(torch.equal(a, b) for a, b in zip(bits, run.raw_results()))
    run.close()


def test_schedule_with_dropout_takes_one_counter_per_forward():
    cfg = SMALL[2]
    n, inflight, seed = 4, 2, 77
    w = syn.make_weights(cfg, sigma=0.05)
    xs, dys = [], []
    for m in range(n):
        x, dy = syn.make_activations(cfg, seed_x=11 + 2 * m, seed_dy=12 + 2 * m)
        xs.append(x); dys.append(dy)
    st = oracle_stage(cfg)
    ref_y, ref_dx, total = [], [], None
    for m in range(n):          # micro-batch m is the m-th forward after set_rng(seed, 100)
        st.set_rng(seed, 100 + m)
        y, dx, g = O.stage_step(st, w, xs[m], dys[m])
        ref_y.append(y); ref_dx.append(dx)
        total = g if total is None else [{k: total[l][k] + g[l][k] for k in g[l]} for l in range(cfg.n_layers)]
    run = ScheduleRunner(cfg, w, xs, dys)
    B.stage_set_rng(run.stage, seed, 100)
    run.poison_outputs()
    run.run(O.one_f_one_b(n, inflight), inflight, syn.plan_swap_ffn_recompute_norm_gelu(cfg))
    ys, dxs, g = run.results()
    bound = 2e-2
    for m in range(n):
        assert O.max_rel_err(ys[m], ref_y[m]) <= bound and O.max_rel_err(dxs[m], ref_dx[m]) <= bound
    for l in range(cfg.n_layers):
        for k in syn.WEIGHT_NAMES:
            assert O.max_rel_err(g[l][k], total[l][k]) <= bound, (l, k)
    run.close()


def test_validator_rejects_bad_rates():
    for kw in (dict(p_attn=1.0), dict(p_hidden=-0.5), dict(p_attn=float("nan"))):
        cfg = dataclasses.replace(SMALL[0], **kw)
        with pytest.raises(B.DpError):
            B.plan_validate(B.make_config(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, cfg.micro_batch,
                                          cfg.norm_style, cfg.causal, cfg.gelu, cfg.dtype, cfg.ln_eps, cfg.p_attn,
                                          cfg.p_hidden), syn.plan_keep_all(cfg))


def test_c2_full_size_with_dropout():
    cfg = dataclasses.replace(syn.CONFIGS["C2"], p_attn=0.1, p_hidden=0.1)
    w = syn.make_weights(cfg)
    x, dy = syn.make_activations(cfg)
    run = StageRunner(cfg, w, x, dy)
    B.stage_set_rng(run.stage, 5, 9)
    run.poison_outputs()
    run.step(syn.plan_keep_all(cfg))
    got, bits = run.results(), run.raw_results()
    st = oracle_stage(cfg)
    st.set_rng(5, 9)
    ref = O.stage_step(st, w, x, dy, dtype=np.float32)
    compare(cfg, got, ref)
    for plan in (syn.plan_all_recompute(cfg), syn.plan_seeded(cfg, 7)):
        B.stage_set_rng(run.stage, 5, 9)
        run.poison_outputs()
        run.step(plan)
        assert all(torch.equal(a, b) for a, b in zip(bits, run.raw_results()))
    run.close()
