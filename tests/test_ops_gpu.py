"""Operator-level parity of the HIP kernels against the CPU oracle, through the
C ABI.  Tolerances: max|gpu-ref| / max|ref| <= 1e-4 in fp32 and <= 2e-2 in bf16
(the bounds the stage step has to meet); most operators are far inside them and
are held to tighter figures derived from one rounding of the output."""
import numpy as np
import pytest
import torch

import synthetic as syn
from oracle import stage as O
from paper_2505_05856_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = {torch.float32: 2e-5, torch.bfloat16: 8e-3}   # one output rounding: 2^-8 relative in bf16


def dev(a, dt):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV).to(dt).contiguous()


def host(t):
    return t.float().cpu().numpy().astype(np.float64)


def rnd(shape, seed, dt, scale=1.0):
    a = scale * syn.normal(seed, 0, int(np.prod(shape))).reshape(shape)
    a = a.astype(np.float32)
    return syn.round_to_bf16(a) if dt == torch.bfloat16 else a


def ws_for(rows, cols):
    return torch.empty(B.op_workspace_bytes(rows, cols), dtype=torch.uint8, device=DEV)


@pytest.mark.parametrize("kind", ["layer", "rms"])
@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("rows,cols", [(1, 8), (7, 16), (130, 128), (37, 1600), (9, 4096), (5, 8192), (2, 2056),
                                       (1301, 4096), (270, 5000), (515, 8192)])
def test_layernorm(dt, rows, cols, kind):
    fwd, bwd = O.NORMS[kind]
    op_fwd, op_bwd = (B.op_layernorm_fwd, B.op_layernorm_bwd) if kind == "layer" else (B.op_rmsnorm_fwd, B.op_rmsnorm_bwd)
    x = rnd((rows, cols), 11, dt, 2.0) + 0.5
    x = syn.round_to_bf16(x) if dt == torch.bfloat16 else x
    g = rnd((cols,), 12, dt) * 0.1 + 1
    g = syn.round_to_bf16(g) if dt == torch.bfloat16 else g
    b = rnd((cols,), 13, dt, 0.1)
    dy = rnd((rows, cols), 14, dt)
    dres = rnd((rows, cols), 15, dt)
    y_ref, mu, r = fwd(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64), 1e-5)
    dx_ref, dg_ref, db_ref = bwd(dy.astype(np.float64), x.astype(np.float64), mu, r, g.astype(np.float64))
    tx, tg, tb, tdy, tres = (dev(a, dt) for a in (x, g, b, dy, dres))
    y = torch.empty_like(tx); stats = torch.empty(rows, 2, dtype=torch.float32, device=DEV)
    op_fwd(tx, tg, tb, 1e-5, y, stats)
    assert O.max_rel_err(host(y), y_ref) < TOL[dt]
    assert np.allclose(host(stats)[:, 0], mu, atol=1e-5) and np.allclose(host(stats)[:, 1], r, rtol=1e-5)
    # stats only / y only
    stats2 = torch.zeros_like(stats)
    op_fwd(tx, tg, tb, 1e-5, None, stats2)
    assert torch.equal(stats, stats2)
    dx = torch.empty_like(tx); dg = torch.empty_like(tg); db = torch.empty_like(tb)
    ws = ws_for(rows, cols)
    op_bwd(tdy, tx, stats, tg, None, dx, dg, db, ws)
    assert O.max_rel_err(host(dx), dx_ref) < TOL[dt]
    assert O.max_rel_err(host(dg), dg_ref) < TOL[dt] and O.max_rel_err(host(db), db_ref) < TOL[dt]
    # with the residual gradient added, written in place over dy
    dy2 = tdy.clone()
    dsum = torch.empty_like(tg)
    op_bwd(dy2, tx, stats, tg, tres, dy2, dg, db, ws, dx_colsum=dsum)
    assert O.max_rel_err(host(dy2), dx_ref + dres) < TOL[dt]
    assert O.max_rel_err(host(dg), dg_ref) < TOL[dt] and O.max_rel_err(host(db), db_ref) < TOL[dt]
    # column sums of dx as stored (a bias gradient): exact sum of the kernel's own output up to fp32 ordering
    assert O.max_rel_err(host(dsum), host(dy2).sum(axis=0)) < TOL[dt]


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("kind", [0, 1, 2])
@pytest.mark.parametrize("rows,cols", [(1237, 8), (77, 1032), (300, 4104)])
def test_gelu(dt, kind, rows, cols):
    """Forward, and the backward kernel the stage runs: dx = dy * gelu'(x) and the column sums of dx as stored."""
    x = rnd((rows, cols), 21, dt, 2.5)
    dy = rnd((rows, cols), 22, dt)
    name = ("erf", "tanh", "relu")[kind]
    tx, tdy = dev(x, dt), dev(dy, dt)
    y = torch.empty_like(tx); dx = torch.empty_like(tx)
    db = torch.empty(cols, dtype=dt, device=DEV)
    ws = ws_for(rows, cols)
    B.op_gelu_fwd(tx, y, kind)
    B.op_gelu_bwd(tdy, tx, dx, db, ws, kind)
    dx_ref = dy * O.gelu_grad(x.astype(np.float64), name)
    assert O.max_rel_err(host(y), O.gelu_fwd(x.astype(np.float64), name)) < TOL[dt]
    assert O.max_rel_err(host(dx), dx_ref) < TOL[dt]
    assert O.max_rel_err(host(db), dx_ref.sum(axis=0)) < TOL[dt]
    db2 = torch.empty_like(db)
    B.op_gelu_bwd(tdy, tx, tdy, db2, ws, kind)     # in place
    assert torch.equal(tdy, dx) and torch.equal(db2, db)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("rows,cols", [(1, 8), (33, 24), (1000, 1600), (4096, 520)])
def test_colsum(dt, rows, cols):
    x = rnd((rows, cols), 31, dt)
    tx = dev(x, dt)
    out = torch.empty(cols, dtype=dt, device=DEV)
    B.op_colsum(tx, out, ws_for(rows, cols))
    assert O.max_rel_err(host(out), x.astype(np.float64).sum(axis=0)) < TOL[dt]


GEMM_SHAPES = [(1, 8, 8), (5, 16, 24), (64, 64, 64), (100, 72, 40), (128, 384, 128), (257, 136, 520),
               (300, 1600, 96), (512, 256, 1024), (1000, 520, 1032), (264, 136, 4104), (2048, 1024, 512),
               (4096, 4096, 192), (3900, 4200, 128),   # these two take the 256x256-tile path
               # ragged edges on each tile size of the LDS-direct kernel, both forms (rows of 8 elements for TN)
               (200, 328, 192), (1096, 1304, 256), (3904, 4200, 128), (3900, 4200, 448)]


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm(dt, mode, M, N, K):
    a = rnd((M, K), 41, dt); b = rnd((K, N), 42, dt)
    bias = rnd((N,), 43, dt); res = rnd((M, N), 44, dt)
    ref = a.astype(np.float64) @ b.astype(np.float64)
    if mode == 0:     # A [M,K], B given as [N,K]
        ta, tb = dev(a, dt), dev(b.T, dt)
    else:             # A given as [K,M], B [K,N]
        ta, tb = dev(a.T, dt), dev(b, dt)
    c = torch.empty(M, N, dtype=dt, device=DEV)
    B.op_gemm(mode, M, N, K, ta, tb, None, None, c)
    assert O.max_rel_err(host(c), ref) < TOL[dt]
    B.op_gemm(mode, M, N, K, ta, tb, dev(bias, dt), dev(res, dt), c)
    assert O.max_rel_err(host(c), ref + bias + res) < TOL[dt]
    # res may be C itself (C += A B): every element is read and written by one lane, once
    c = dev(res, dt)
    B.op_gemm(mode, M, N, K, ta, tb, None, c, c)
    assert O.max_rel_err(host(c), ref + res) < TOL[dt]


ATTN_SHAPES = [(1, 8, 1, 8), (2, 5, 2, 16), (2, 64, 2, 64), (1, 200, 3, 64), (2, 96, 2, 128), (1, 384, 2, 64),
               (1, 1024, 3, 64), (1, 2048, 2, 128)]     # the last two: sequence and head width of C3/C4 and of C5


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Bn,S,nh,dh", ATTN_SHAPES)
@pytest.mark.parametrize("sharp", [False, True])
def test_attention(dt, causal, Bn, S, nh, dh, sharp):
    H = nh * dh
    qkv = rnd((Bn * S, 3 * H), 51, dt)
    if sharp:     # logits with a standard deviation of a few units
        qkv[:, :2 * H] *= 2.0
        qkv = syn.round_to_bf16(qkv) if dt == torch.bfloat16 else qkv
    d_o = rnd((Bn * S, H), 52, dt)
    q64 = qkv.astype(np.float64)
    o_ref, lse_ref = O.attention_fwd(q64, Bn, S, nh, causal)
    dq_ref = O.attention_bwd(d_o.astype(np.float64), q64, Bn, S, nh, causal)
    tq, tdo = dev(qkv, dt), dev(d_o, dt)
    o = torch.empty(Bn * S, H, dtype=dt, device=DEV)
    lse = torch.empty(Bn, nh, S, dtype=torch.float32, device=DEV)
    B.op_attention_fwd(tq, Bn, S, nh, dh, causal, o, lse)
    tol = TOL[dt] * (2 if dt == torch.bfloat16 else 1)     # P is rounded to bf16 as well
    assert O.max_rel_err(host(o), o_ref) < tol
    assert np.allclose(host(lse), lse_ref, atol=2e-5 if dt == torch.float32 else 2e-3)
    # single outputs
    lse2 = torch.zeros_like(lse)
    B.op_attention_fwd(tq, Bn, S, nh, dh, causal, None, lse2)
    assert torch.equal(lse, lse2)
    dqkv = torch.empty_like(tq)
    ws = ws_for(Bn * S, nh)
    # the backward is fed the oracle-consistent O the kernel itself produced
    B.op_attention_bwd(tq, o, lse, tdo, Bn, S, nh, dh, causal, dqkv, ws)
    got = host(dqkv)
    for blk in range(3):
        assert O.max_rel_err(got[:, blk * H:(blk + 1) * H], dq_ref[:, blk * H:(blk + 1) * H]) < 2 * tol, blk


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("dh", [64, 128])
def test_attention_with_a_maximum_that_creeps_and_then_jumps(dt, dh):
    """Logits that grow by about two units per 64-key tile, with a jump of thirty for every other query late in
    the row: the forward kernel's reference point for the exponents follows the maximum with a lag, and O and
    the log-sum-exp must not depend on where it stood (the softmax is invariant under the shift)."""
    Bn, S, nh = 1, 1024, 2
    H = nh * dh
    rng = np.random.default_rng(77)
    u = rng.standard_normal(dh); u /= np.linalg.norm(u)
    q = np.tile(u * np.sqrt(dh), (S, 1)) + 0.05 * rng.standard_normal((S, dh))    # q.k / sqrt(dh) = the key's ramp
    ramp = 2.0 * np.arange(S) / 64.0
    k = ramp[:, None] * u[None, :] + 0.05 * rng.standard_normal((S, dh))
    k[700] += 30.0 * u                      # one key far above the ramp ...
    q[0::2] *= 1.0; q[1::2] *= 0.25         # ... by thirty units for even queries, by a quarter of that for odd ones
    v = rng.standard_normal((S, dh))
    qkv = np.zeros((Bn * S, 3 * H))
    for h in range(nh):
        qkv[:, h * dh:(h + 1) * dh] = q
        qkv[:, H + h * dh:H + (h + 1) * dh] = k
        qkv[:, 2 * H + h * dh:2 * H + (h + 1) * dh] = v * (h + 1)
    qkv = syn.round_to_bf16(qkv.astype(np.float32)) if dt == torch.bfloat16 else qkv.astype(np.float32)
    d_o = rnd((Bn * S, H), 78, dt)
    q64 = qkv.astype(np.float64)
    for causal in (False, True):
        o_ref, lse_ref = O.attention_fwd(q64, Bn, S, nh, causal)
        dq_ref = O.attention_bwd(d_o.astype(np.float64), q64, Bn, S, nh, causal)
        tq, tdo = dev(qkv, dt), dev(d_o, dt)
        o = torch.empty(Bn * S, H, dtype=dt, device=DEV)
        lse = torch.empty(Bn, nh, S, dtype=torch.float32, device=DEV)
        B.op_attention_fwd(tq, Bn, S, nh, dh, causal, o, lse)
        tol = TOL[dt] * (2 if dt == torch.bfloat16 else 1)
        assert O.max_rel_err(host(o), o_ref) < tol
        assert np.allclose(host(lse), lse_ref, atol=2e-5 * 40 if dt == torch.float32 else 2e-3 * 40)   # lse reaches ~60
        dqkv = torch.empty_like(tq)
        B.op_attention_bwd(tq, o, lse, tdo, Bn, S, nh, dh, causal, dqkv, ws_for(Bn * S, nh))
        got = host(dqkv)
        for blk in range(3):
            assert O.max_rel_err(got[:, blk * H:(blk + 1) * H], dq_ref[:, blk * H:(blk + 1) * H]) < 2 * tol, (causal, blk)


def test_mfma_issue_probe_reports_a_plausible_rate():
    """The diagnostic behind the roofline discussion: rate = CUs * 4096 flop/clk * clock, so the two numbers it
    returns must agree with each other, and zeros must not run slower than random mantissas."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    zeros = torch.zeros(1 << 16, dtype=torch.bfloat16, device=DEV)
    noise = torch.randint(-2 ** 15, 2 ** 15, (1 << 16,), dtype=torch.int16, device=DEV).view(torch.bfloat16)
    tz, fz = B.probe_mfma(zeros, 20000)
    tn, fn = B.probe_mfma(noise, 20000)
    for t, f in ((tz, fz), (tn, fn)):
        assert 500 < f < 3000
        assert abs(t * 1e12 - cus * 4096 * f * 1e6) <= 0.25 * t * 1e12     # one CU's clock; launch and drain included
    assert tz >= 0.98 * tn
    with pytest.raises(B.DpError):
        B.probe_mfma(zeros[:4], 10)


@pytest.mark.parametrize("mode,M,N,K", [(0, 4096, 4096, 4096), (0, 4096, 4096, 11008), (0, 3072, 1600, 6400),
                                        (1, 4096, 4096, 16384), (1, 1600, 6400, 32768), (1, 4096, 11008, 8192)])
def test_gemm_long_contractions_of_the_wide_configurations(mode, M, N, K):
    """The contraction lengths of C4/C5 (hidden 4096, ffn 11008; weight gradients over 16384 and 32768 tokens) at
    output sizes that take the 256x256 tiles and their five-tile ring, against a float32 reference product (its
    own rounding, ~K * 6e-8 relative, is far below one bf16 rounding of the output)."""
    dt = torch.bfloat16
    a = rnd((M, K), 91, dt, 0.5); b = rnd((K, N), 92, dt, 0.5)
    ref = a @ b                                  # float32 in, float32 out
    ta, tb = (dev(a, dt), dev(np.ascontiguousarray(b.T), dt)) if mode == 0 else (dev(np.ascontiguousarray(a.T), dt), dev(b, dt))
    c = torch.empty(M, N, dtype=dt, device=DEV)
    B.op_gemm(mode, M, N, K, ta, tb, None, None, c)
    got = c.float().cpu().numpy()
    scale = np.abs(ref).max()
    assert np.abs(got - ref).max() <= TOL[dt] * scale
    # every 4096th element exactly as one rounding of the float64 product of that row and column
    rows = np.arange(0, M, 509)[:6]; cols = np.arange(0, N, 613)[:6]
    exact = a[rows].astype(np.float64) @ b[:, cols].astype(np.float64)
    assert np.abs(got[np.ix_(rows, cols)] - exact).max() <= 2.0 ** -8 * np.abs(exact).max() + 1e-6


# The column reductions at the token counts of the wide configurations (C5: 16384 tokens, C4: 32768): above 4096
# (LayerNorm backward) or 8192 rows (the other two) a row block of the two-pass reductions covers more than its
# minimum number of rows, a regime the smaller shapes above never enter.
@pytest.mark.parametrize("rows", [16384, 32768])
@pytest.mark.parametrize("cols", [1600, 4096])
def test_layernorm_backward_over_many_rows(rows, cols):
    dt = torch.bfloat16
    fwd, bwd = O.NORMS["layer"]
    x = syn.round_to_bf16(rnd((rows, cols), 11, dt, 2.0) + 0.5)
    g = syn.round_to_bf16(rnd((cols,), 12, dt) * 0.1 + 1)
    b = rnd((cols,), 13, dt, 0.1)
    dy = rnd((rows, cols), 14, dt)
    dres = rnd((rows, cols), 15, dt)
    x64, g64 = x.astype(np.float64), g.astype(np.float64)
    _, mu, r = fwd(x64, g64, b.astype(np.float64), 1e-5)
    dx_ref, dg_ref, db_ref = bwd(dy.astype(np.float64), x64, mu, r, g64)
    tx, tg, tdy, tres = (dev(a, dt) for a in (x, g, dy, dres))
    stats = torch.from_numpy(np.stack([mu, r], axis=1).astype(np.float32)).to(DEV)
    dx = torch.empty_like(tx); dgo = torch.empty_like(tg); dbo = torch.empty_like(tg); dsum = torch.empty_like(tg)
    B.op_layernorm_bwd(tdy, tx, stats, tg, tres, dx, dgo, dbo, ws_for(rows, cols), dx_colsum=dsum)
    assert O.max_rel_err(host(dx), dx_ref + dres) < TOL[dt]
    assert O.max_rel_err(host(dgo), dg_ref) < TOL[dt] and O.max_rel_err(host(dbo), db_ref) < TOL[dt]
    assert O.max_rel_err(host(dsum), host(dx).sum(axis=0)) < TOL[dt]


@pytest.mark.parametrize("rows", [16384, 32768])
@pytest.mark.parametrize("cols", [1600, 6400])
def test_gelu_backward_and_column_sums_over_many_rows(rows, cols):
    dt = torch.bfloat16
    x = rnd((rows, cols), 21, dt, 2.5)
    dy = rnd((rows, cols), 22, dt)
    tx, tdy = dev(x, dt), dev(dy, dt)
    dx = torch.empty_like(tx)
    db = torch.empty(cols, dtype=dt, device=DEV)
    ws = ws_for(rows, cols)
    B.op_gelu_bwd(tdy, tx, dx, db, ws, 0)
    dx_ref = dy * O.gelu_grad(x.astype(np.float64), "erf")
    assert O.max_rel_err(host(dx), dx_ref) < TOL[dt]
    assert O.max_rel_err(host(db), dx_ref.sum(axis=0)) < TOL[dt]
    out = torch.empty(cols, dtype=dt, device=DEV)
    B.op_colsum(tx, out, ws)
    assert O.max_rel_err(host(out), x.astype(np.float64).sum(axis=0)) < TOL[dt]
