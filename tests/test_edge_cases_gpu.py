"""Edge cases through the C ABI: empty inputs, the smallest and the largest extents the kernels
take, degenerate attention (one key), and the smallest stage."""
import numpy as np
import pytest
import torch

import synthetic as syn
from oracle import stage as O
from paper_2505_05856_amd import binding as B
from paper_2505_05856_amd.harness import StageRunner
from test_ops_gpu import DEV, TOL, dev, host, rnd, ws_for
from test_stage_gpu import compare, oracle_step

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_empty_inputs_are_no_ops_and_empty_sums_are_zero(dt):
    cols = 64
    # zero-row views of real storage: an empty torch tensor of its own has a null pointer, which the
    # library rejects as a missing argument
    e = torch.zeros(1, cols, dtype=dt, device=DEV)[:0]
    g = torch.ones(cols, dtype=dt, device=DEV)
    stats = torch.zeros(1, 2, dtype=torch.float32, device=DEV)[:0]
    nan = lambda: torch.full((cols,), float("nan"), dtype=dt, device=DEV)
    ws = ws_for(8, cols)
    B.op_layernorm_fwd(e, g, g, 1e-5, torch.zeros(1, cols, dtype=dt, device=DEV)[:0], stats)
    dg, db, ds = nan(), nan(), nan()
    B.op_layernorm_bwd(e, e, stats, g, None, torch.zeros(1, cols, dtype=dt, device=DEV)[:0], dg, db, ws, dx_colsum=ds)
    out = nan()
    B.op_colsum(e, out, ws)
    torch.cuda.synchronize()
    for t in (dg, db, ds, out):
        assert torch.equal(t, torch.zeros_like(t))
    # the same for the other normalisation
    B.op_rmsnorm_fwd(e, g, g, 1e-5, torch.zeros(1, cols, dtype=dt, device=DEV)[:0], stats)
    dg, db, ds = nan(), nan(), nan()
    B.op_rmsnorm_bwd(e, e, stats, g, None, torch.zeros(1, cols, dtype=dt, device=DEV)[:0], dg, db, ws, dx_colsum=ds)
    torch.cuda.synchronize()
    for t in (dg, db, ds):
        assert torch.equal(t, torch.zeros_like(t))
    B.op_gelu_fwd(e, torch.zeros(1, cols, dtype=dt, device=DEV)[:0])
    out = nan()
    B.op_gelu_bwd(e, e, torch.zeros(1, cols, dtype=dt, device=DEV)[:0], out, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, torch.zeros_like(out))
    # GEMM with an empty extent: nothing to write; K = 0: the product is zero, bias and residual remain
    a = torch.zeros(1, 64, dtype=dt, device=DEV)[:0]
    b = dev(rnd((128, 64), 3, dt), dt)
    B.op_gemm(0, 0, 128, 64, a, b, None, None, torch.zeros(1, 128, dtype=dt, device=DEV)[:0])
    bias, res = rnd((128,), 4, dt), rnd((8, 128), 5, dt)
    c = torch.full((8, 128), float("nan"), dtype=dt, device=DEV)
    B.op_gemm(0, 8, 128, 0, torch.zeros(8, 1, dtype=dt, device=DEV)[:, :0], torch.zeros(128, 1, dtype=dt, device=DEV)[:, :0],
              dev(bias, dt), dev(res, dt), c)
    assert O.max_rel_err(host(c), res.astype(np.float64) + bias) < TOL[dt]
    # attention over no sequences
    B.op_attention_fwd(torch.zeros(1, 192, dtype=dt, device=DEV)[:0], 0, 16, 1, 64, False,
                       torch.zeros(1, 64, dtype=dt, device=DEV)[:0], torch.zeros(1, 1, 16, dtype=torch.float32, device=DEV)[:0])
    torch.cuda.synchronize()


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("dh", [8, 64, 128])
def test_attention_with_one_key_returns_the_value(dt, dh):
    """S = 1 (and row 0 of any causal problem): the softmax over one key is 1, O = V, LSE = the logit,
    dV = dO, dQ = dK = 0."""
    Bn, nh = 3, 2
    H = nh * dh
    qkv = rnd((Bn, 3 * H), 71, dt)
    d_o = rnd((Bn, H), 72, dt)
    tq, tdo = dev(qkv, dt), dev(d_o, dt)
    o = torch.empty(Bn, H, dtype=dt, device=DEV)
    lse = torch.empty(Bn, nh, 1, dtype=torch.float32, device=DEV)
    B.op_attention_fwd(tq, Bn, 1, nh, dh, True, o, lse)
    assert torch.equal(o, tq[:, 2 * H:])
    logit = (qkv[:, :H].reshape(Bn, nh, dh).astype(np.float64) * qkv[:, H:2 * H].reshape(Bn, nh, dh)).sum(-1) / np.sqrt(dh)
    assert np.allclose(host(lse)[:, :, 0], logit, atol=2e-3 if dt == torch.bfloat16 else 1e-5)
    dqkv = torch.empty_like(tq)
    B.op_attention_bwd(tq, o, lse, tdo, Bn, 1, nh, dh, True, dqkv, ws_for(Bn, nh))
    got = host(dqkv)
    assert np.array_equal(got[:, 2 * H:], host(tdo))
    assert np.abs(got[:, :2 * H]).max() <= (2e-2 if dt == torch.bfloat16 else 1e-5) * np.abs(host(tdo)).max()


def test_longest_sequence_of_the_vector_kernels_and_beyond_on_the_matrix_cores():
    """fp32 attention keeps a row of scores in LDS: 4096 keys is its limit and 4097 an error; the bf16 matrix-core
    kernels go on (8192 keys here), checked on sampled rows against the oracle's softmax written per row."""
    S, dh = 4096, 64
    qkv = rnd((S, 3 * dh), 81, torch.float32)
    tq = dev(qkv, torch.float32)
    o = torch.empty(S, dh, dtype=torch.float32, device=DEV)
    lse = torch.empty(1, 1, S, dtype=torch.float32, device=DEV)
    B.op_attention_fwd(tq, 1, S, 1, dh, False, o, lse)
    ref, _ = O.attention_fwd(qkv.astype(np.float64), 1, S, 1, False)
    assert O.max_rel_err(host(o), ref) < TOL[torch.float32]
    with pytest.raises(B.DpError) as e:
        B.op_attention_fwd(dev(rnd((S + 1, 3 * dh), 82, torch.float32), torch.float32), 1, S + 1, 1, dh, False,
                           torch.empty(S + 1, dh, dtype=torch.float32, device=DEV), None)
    assert e.value.status == "DP_E_UNSUPPORTED"
    S = 8192
    qkv = rnd((S, 3 * dh), 83, torch.bfloat16)
    tq = dev(qkv, torch.bfloat16)
    o = torch.empty(S, dh, dtype=torch.bfloat16, device=DEV)
    B.op_attention_fwd(tq, 1, S, 1, dh, True, o, None)
    q64 = qkv.astype(np.float64)
    got = host(o)
    for i in (0, 1, 63, 64, 4095, 4096, 8000, S - 1):
        a = q64[i, :dh] @ q64[:i + 1, dh:2 * dh].T / np.sqrt(dh)
        p = np.exp(a - a.max()); p /= p.sum()
        assert np.abs(got[i] - p @ q64[:i + 1, 2 * dh:]).max() <= 2e-2 * np.abs(q64[:, 2 * dh:]).max(), i


def test_the_smallest_stage():
    """One layer, one sequence of one token, one head of width 8."""
    for style in ("pre", "post"):
        for dtype in ("f32", "bf16"):
            cfg = syn.StageConfig(1, 8, 1, 8, 1, 1, style, True, "erf", dtype)
            w = syn.make_weights(cfg, sigma=0.3)
            x, dy = syn.make_activations(cfg)
            run = StageRunner(cfg, w, x, dy)
            ref = oracle_step(cfg, w, x, dy)
            bits = []
            for plan in (syn.plan_keep_all(cfg), syn.plan_all_recompute(cfg), syn.plan_all_swap(cfg)):
                run.poison_outputs()
                run.step(plan)
                compare(cfg, run.results(), ref, bound=3e-2 if dtype == "bf16" else None)
                bits.append(run.raw_results())
            assert all(torch.equal(a, b) for a, b in zip(bits[0], bits[1])) and \
                   all(torch.equal(a, b) for a, b in zip(bits[0], bits[2]))
            run.close()


def test_fallback_launches_are_counted_in_the_step_statistics():
    """A head dimension the matrix-core attention does not take: the step runs (vector-ALU kernels), matches the
    oracle, and says so in its statistics; a supported shape reports none."""
    for cfg, want in ((syn.StageConfig(2, 192, 2, 384, 64, 2, "pre", True, "erf", "bf16"), 4),
                      (syn.StageConfig(2, 128, 2, 256, 64, 2, "pre", True, "erf", "bf16"), 0)):
        w = syn.make_weights(cfg)
        x, dy = syn.make_activations(cfg)
        run = StageRunner(cfg, w, x, dy)
        stats = run.step(syn.plan_keep_all(cfg), want_stats=True)
        assert stats["n_fallback_launches"] == want
        assert stats["replay_ms"] == 0.0 and stats["d2h_busy_ms"] == 0.0 and stats["swap_wait_ms"] == 0.0
        compare(cfg, run.results(), oracle_step(cfg, w, x, dy))
        stats = run.step(syn.plan_all_swap(cfg), want_stats=True)
        assert stats["d2h_busy_ms"] > 0.0 and stats["h2d_busy_ms"] > 0.0 and stats["d2h_bytes"] == stats["h2d_bytes"] > 0
        stats = run.step(syn.plan_all_recompute(cfg), want_stats=True)
        assert stats["replay_ms"] > 0.0 and stats["n_replayed_ops"] > 0
        run.close()
