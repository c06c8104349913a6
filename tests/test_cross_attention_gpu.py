"""Cross-attention on the device against the CPU oracle, through the C ABI: queries of one
sequence over keys and values of another, lengths that span several 128-row and 64-key tiles
with ragged tails, both head dimensions of the matrix-core kernels and the vector kernels
(fp32), sharp logits, dropout with the oracle's mask, empty sides, and the self-attention
entry point as the special case it is (bit for bit).  Bounds: max|gpu-ref| / max|ref| against
one output rounding (doubled where the probabilities are rounded to bf16 as well)."""
import warnings

import numpy as np
import pytest
import torch

import synthetic as syn
from oracle import dropout as D
from oracle import stage as O
from paper_2505_05856_amd import binding as B
from test_ops_gpu import DEV, TOL, dev, host, rnd, ws_for

pytestmark = pytest.mark.gpu
warnings.filterwarnings("ignore", message="overflow encountered")

SHAPES = [  # B, Sq, Sk, nh, dh
    (2, 5, 3, 2, 64), (1, 1, 1, 1, 64), (2, 37, 130, 2, 64), (1, 300, 77, 3, 64), (2, 129, 64, 1, 128),
    (1, 70, 257, 2, 128), (1, 256, 512, 2, 64), (3, 64, 1, 2, 64), (1, 1, 200, 2, 128), (2, 40, 24, 2, 16)]


def run_case(dt, Bn, Sq, Sk, nh, dh, sharp=False, drop=None):
    H = nh * dh
    q, kv, d_o = rnd((Bn * Sq, H), 71, dt), rnd((Bn * Sk, 2 * H), 72, dt), rnd((Bn * Sq, H), 73, dt)
    if sharp:     # logits with a standard deviation of a few units
        q, kv = q * 2.0, kv.copy()
        kv[:, :H] *= 2.0
        if dt == torch.bfloat16:
            q, kv = syn.round_to_bf16(q), syn.round_to_bf16(kv)
    keep, scale, bd = None, 1.0, None
    if drop is not None:
        p, seed, mb, layer = drop
        masks = [D.keep_cross_attention(seed, mb, layer, b, nh, Sq, Sk, p) for b in range(Bn)]
        keep, scale, bd = (lambda b: masks[b]), D.scale(p), B.Dropout(p, seed, mb, layer)
    q64, kv64 = q.astype(np.float64), kv.astype(np.float64)
    o_ref, lse_ref = O.cross_attention_fwd(q64, kv64, Bn, Sq, Sk, nh, keep, scale)
    dq_ref, dkv_ref = O.cross_attention_bwd(d_o.astype(np.float64), q64, kv64, Bn, Sq, Sk, nh, keep, scale)
    tq, tkv, tdo = dev(q, dt), dev(kv, dt), dev(d_o, dt)
    o = torch.empty(Bn * Sq, H, dtype=dt, device=DEV)
    lse = torch.empty(Bn, nh, Sq, dtype=torch.float32, device=DEV)
    B.op_cross_attention_fwd(tq, tkv, Bn, Sq, Sk, nh, dh, o, lse, bd)
    tol = TOL[dt] * (2 if dt == torch.bfloat16 else 1)     # P is rounded to bf16 as well
    assert O.max_rel_err(host(o), o_ref) < tol
    assert np.allclose(host(lse), lse_ref, atol=2e-5 if dt == torch.float32 else 2e-3)
    lse2 = torch.zeros_like(lse)
    B.op_cross_attention_fwd(tq, tkv, Bn, Sq, Sk, nh, dh, None, lse2, bd)
    assert torch.equal(lse, lse2)
    dq = torch.full_like(tq, float("nan")); dkv = torch.full_like(tkv, float("nan"))
    B.op_cross_attention_bwd(tq, tkv, o, lse, tdo, Bn, Sq, Sk, nh, dh, dq, dkv, ws_for(Bn * Sq, nh), bd)
    assert O.max_rel_err(host(dq), dq_ref) < 2 * tol or np.abs(dq_ref).max() < 1e-12 and np.abs(host(dq)).max() < 1e-6
    assert O.max_rel_err(host(dkv)[:, :H], dkv_ref[:, :H]) < 2 * tol or (
        np.abs(dkv_ref[:, :H]).max() < 1e-12 and np.abs(host(dkv)[:, :H]).max() < 1e-6)
    assert O.max_rel_err(host(dkv)[:, H:], dkv_ref[:, H:]) < 2 * tol
    return o, lse, dq, dkv


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", SHAPES)
def test_cross_attention(dt, shape):
    run_case(dt, *shape)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", [(2, 37, 130, 2, 64), (1, 70, 257, 2, 128)])
def test_sharp_logits(dt, shape):
    run_case(dt, *shape, sharp=True)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", [(2, 37, 130, 2, 64), (1, 150, 70, 2, 128), (2, 5, 3, 2, 64)])
@pytest.mark.parametrize("p", [0.1, 0.5])
def test_dropout_with_the_oracles_mask(dt, shape, p):
    run_case(dt, *shape, drop=(p, 0xABCDEF0123456789, 3 + (1 << 33), 2))


def test_the_mask_bits_are_the_oracles():
    """V = identity columns makes O row i the masked, scaled probabilities themselves: with equal keys the
    probabilities are uniform, so O * Sk / scale is exactly the keep mask."""
    Bn, Sq, Sk, nh, dh, p = 2, 70, 64, 2, 64, 0.3
    H = nh * dh
    q = rnd((Bn * Sq, H), 1, torch.float32)
    kv = np.zeros((Bn * Sk, 2 * H), dtype=np.float32)
    for b in range(Bn):
        for h in range(nh):
            kv[b * Sk:(b + 1) * Sk, H + h * dh:H + (h + 1) * dh] = np.eye(Sk, dh)
    for dt in (torch.float32, torch.bfloat16):
        o = torch.empty(Bn * Sq, H, dtype=dt, device=DEV)
        B.op_cross_attention_fwd(dev(q, dt), dev(kv, dt), Bn, Sq, Sk, nh, dh, o, None, B.Dropout(p, 77, 5, 1))
        got = host(o).reshape(Bn, Sq, nh, dh).transpose(0, 2, 1, 3) != 0
        for b in range(Bn):
            assert np.array_equal(got[b], D.keep_cross_attention(77, 5, 1, b, nh, Sq, Sk, p))


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("Bn,S,nh,dh", [(2, 200, 2, 64), (1, 130, 2, 128)])
def test_self_attention_is_the_special_case_bit_for_bit(dt, Bn, S, nh, dh):
    H = nh * dh
    qkv = rnd((Bn * S, 3 * H), 81, dt); d_o = rnd((Bn * S, H), 82, dt)
    tqkv, tdo = dev(qkv, dt), dev(d_o, dt)
    o = torch.empty(Bn * S, H, dtype=dt, device=DEV); lse = torch.empty(Bn, nh, S, dtype=torch.float32, device=DEV)
    B.op_attention_fwd(tqkv, Bn, S, nh, dh, False, o, lse)
    dqkv = torch.empty_like(tqkv)
    B.op_attention_bwd(tqkv, o, lse, tdo, Bn, S, nh, dh, False, dqkv, ws_for(Bn * S, nh))
    tq, tkv = tqkv[:, :H].contiguous(), tqkv[:, H:].contiguous()
    o2 = torch.empty_like(o); lse2 = torch.empty_like(lse)
    B.op_cross_attention_fwd(tq, tkv, Bn, S, S, nh, dh, o2, lse2)
    dq = torch.empty_like(tq); dkv = torch.empty_like(tkv)
    B.op_cross_attention_bwd(tq, tkv, o2, lse2, tdo, Bn, S, S, nh, dh, dq, dkv, ws_for(Bn * S, nh))
    assert torch.equal(o, o2) and torch.equal(lse, lse2)
    assert torch.equal(dqkv[:, :H], dq) and torch.equal(dqkv[:, H:], dkv)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_empty_sides_and_bad_arguments(dt):
    nh, dh = 2, 64
    H = nh * dh
    one = torch.ones(1, dtype=dt, device=DEV)     # a valid pointer for tensors without elements
    # no queries: forward writes nothing; backward writes dkv = 0
    kv = dev(rnd((2 * 9, 2 * H), 3, dt), dt)
    B.op_cross_attention_fwd(one, kv, 2, 0, 9, nh, dh, one, None)
    dkv = torch.full_like(kv, float("nan"))
    B.op_cross_attention_bwd(one, kv, one, one.float(), one, 2, 0, 9, nh, dh, one, dkv, ws_for(1, nh))
    assert torch.count_nonzero(dkv) == 0
    # no samples at all
    B.op_cross_attention_fwd(one, one, 0, 4, 4, nh, dh, one, None)
    # queries without keys, a head dimension that is no multiple of 8, negative extents
    q = dev(rnd((4, H), 4, dt), dt)
    o = torch.empty_like(q)
    for args in ((1, 4, 0, nh, dh), (1, 4, 4, nh, 12), (1, -1, 4, nh, dh), (1, 4, -4, nh, dh)):
        with pytest.raises(B.DpError):
            B.op_cross_attention_fwd(q, kv, *args, o, None)
    with pytest.raises(B.DpError):
        B.op_cross_attention_fwd(q, kv, 1, 4, 4, nh, dh, o, None, B.Dropout(1.0, 1, 1, 0))
    if dt == torch.bfloat16:    # the matrix-core kernels store 16 bytes a lane: an output 2 bytes off is refused, nothing runs
        off = torch.zeros(4 * H + 1, dtype=dt, device=DEV)
        with pytest.raises(B.DpError):
            B.op_cross_attention_fwd(q, kv, 1, 4, 4, nh, dh, off[1:].view(4, H), None)
        assert torch.count_nonzero(off) == 0
