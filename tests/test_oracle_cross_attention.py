"""Pins for the oracle's cross-attention (queries of one sequence over keys and values of
another; the paper names T5 in Section 5.1 and gives no formulas): element-by-element loops,
closed forms, the self-attention special case, invariances, central differences and torch
autograd.  A dropped 1/sqrt(dh), a transposed operand, K and V swapped or a wrong sample
offset on either side fails at least one of them."""
import math

import numpy as np
import pytest

from oracle import dropout as D
from oracle import stage as O

rng = np.random.default_rng(11)


def _brute(q, kv, B, Sq, Sk, nh, keep=None, scale=1.0):
    H = q.shape[1]
    dh = H // nh
    out = np.zeros((B * Sq, H))
    lse = np.zeros((B, nh, Sq))
    for b in range(B):
        for h in range(nh):
            for i in range(Sq):
                qv = q[b * Sq + i, h * dh:(h + 1) * dh]
                sc = [sum(qv[d] * kv[b * Sk + j, h * dh + d] for d in range(dh)) / math.sqrt(dh) for j in range(Sk)]
                z = sum(math.exp(s) for s in sc)
                lse[b, h, i] = math.log(z)
                for d in range(dh):
                    out[b * Sq + i, h * dh + d] = sum(
                        math.exp(sc[j]) / z * (1.0 if keep is None else keep[b][h, i, j] * scale)
                        * kv[b * Sk + j, H + h * dh + d] for j in range(Sk))
    return out, lse


@pytest.mark.parametrize("Sq,Sk", [(5, 3), (2, 7), (1, 1)])
def test_fwd_element_by_element(Sq, Sk):
    B, nh, dh = 2, 2, 4
    q = rng.normal(size=(B * Sq, nh * dh)); kv = rng.normal(size=(B * Sk, 2 * nh * dh))
    o, lse = O.cross_attention_fwd(q, kv, B, Sq, Sk, nh)
    o2, lse2 = _brute(q, kv, B, Sq, Sk, nh)
    assert np.allclose(o, o2, atol=1e-12) and np.allclose(lse, lse2, atol=1e-12)


def test_self_attention_is_the_special_case():
    B, S, nh, dh = 2, 6, 3, 4
    H = nh * dh
    qkv = rng.normal(size=(B * S, 3 * H)); do = rng.normal(size=(B * S, H))
    q, kv = np.ascontiguousarray(qkv[:, :H]), np.ascontiguousarray(qkv[:, H:])
    o, lse = O.cross_attention_fwd(q, kv, B, S, S, nh)
    o2, lse2 = O.attention_fwd(qkv, B, S, nh, False)
    assert np.allclose(o, o2, atol=1e-13) and np.allclose(lse, lse2, atol=1e-13)
    dq, dkv = O.cross_attention_bwd(do, q, kv, B, S, S, nh)
    d2 = O.attention_bwd(do, qkv, B, S, nh, False)
    assert np.allclose(dq, d2[:, :H], atol=1e-13) and np.allclose(dkv, d2[:, H:], atol=1e-13)


def test_closed_forms():
    B, Sq, nh, dh = 2, 4, 2, 4
    H = nh * dh
    q = rng.normal(size=(B * Sq, H)); do = rng.normal(size=(B * Sq, H))
    # one key: every query returns that sample's value row; lse is the single logit; the
    # softmax is constant, so nothing flows to Q or K and dV is the sum of dO over the queries
    kv = rng.normal(size=(B, 2 * H))
    o, lse = O.cross_attention_fwd(q, kv, B, Sq, 1, nh)
    for b in range(B):
        assert np.allclose(o[b * Sq:(b + 1) * Sq], kv[b, H:])
        for h in range(nh):
            logit = q[b * Sq:(b + 1) * Sq, h * dh:(h + 1) * dh] @ kv[b, h * dh:(h + 1) * dh] / math.sqrt(dh)
            assert np.allclose(lse[b, h], logit)
    dq, dkv = O.cross_attention_bwd(do, q, kv, B, Sq, 1, nh)
    assert np.allclose(dq, 0, atol=1e-13) and np.allclose(dkv[:, :H], 0, atol=1e-13)
    assert np.allclose(dkv[:, H:], do.reshape(B, Sq, H).sum(axis=1))
    # equal keys: uniform weights, the mean of the values, lse = logit + log(Sk)
    Sk = 5
    kv = rng.normal(size=(B * Sk, 2 * H))
    kv[:, :H] = np.repeat(kv[::Sk, :H], Sk, axis=0)
    o, lse = O.cross_attention_fwd(q, kv, B, Sq, Sk, nh)
    for b in range(B):
        assert np.allclose(o[b * Sq:(b + 1) * Sq], kv[b * Sk:(b + 1) * Sk, H:].mean(axis=0))
    o1, lse1 = O.cross_attention_fwd(q, kv[::Sk].copy(), B, Sq, 1, nh)
    assert np.allclose(lse, lse1 + math.log(Sk))


def test_key_order_and_sample_independence():
    B, Sq, Sk, nh, dh = 2, 3, 6, 2, 4
    H = nh * dh
    q = rng.normal(size=(B * Sq, H)); kv = rng.normal(size=(B * Sk, 2 * H)); do = rng.normal(size=(B * Sq, H))
    o, lse = O.cross_attention_fwd(q, kv, B, Sq, Sk, nh)
    dq, dkv = O.cross_attention_bwd(do, q, kv, B, Sq, Sk, nh)
    perm = rng.permutation(Sk)
    rows = np.concatenate([b * Sk + perm for b in range(B)])
    o2, lse2 = O.cross_attention_fwd(q, kv[rows], B, Sq, Sk, nh)
    dq2, dkv2 = O.cross_attention_bwd(do, q, kv[rows], B, Sq, Sk, nh)
    assert np.allclose(o, o2, atol=1e-13) and np.allclose(lse, lse2, atol=1e-13)
    assert np.allclose(dq, dq2, atol=1e-13) and np.allclose(dkv[rows], dkv2, atol=1e-13)
    # sample 1's keys do not reach sample 0's queries
    kv3 = kv.copy(); kv3[Sk:] = rng.normal(size=(Sk, 2 * H))
    o3, _ = O.cross_attention_fwd(q, kv3, B, Sq, Sk, nh)
    assert np.array_equal(o3[:Sq], o[:Sq]) and not np.allclose(o3[Sq:], o[Sq:])
    # a constant added to every key moves each row's logits together: O and dQ-side unchanged, sum_j dK_j = 0
    assert np.allclose(dkv[:Sk, :H].sum(axis=0), 0, atol=1e-12)


def test_backward_central_differences():
    B, Sq, Sk, nh, dh = 2, 3, 5, 2, 4
    H = nh * dh
    q = rng.normal(size=(B * Sq, H)); kv = rng.normal(size=(B * Sk, 2 * H)); do = rng.normal(size=(B * Sq, H))
    keep = [D.keep_cross_attention(5, 2, 1, b, nh, Sq, Sk, 0.3) for b in range(B)]
    for kf, sc in ((None, 1.0), (lambda b: keep[b], D.scale(0.3))):
        f = lambda q_, kv_: float((O.cross_attention_fwd(q_, kv_, B, Sq, Sk, nh, kf, sc)[0] * do).sum())
        dq, dkv = O.cross_attention_bwd(do, q, kv, B, Sq, Sk, nh, kf, sc)
        eps = 1e-6
        for arr, grad, which in ((q, dq, 0), (kv, dkv, 1)):
            num = np.zeros_like(arr)
            for idx in np.ndindex(arr.shape):
                a = arr.copy(); a[idx] += eps
                b_ = arr.copy(); b_[idx] -= eps
                num[idx] = ((f(a, kv) - f(b_, kv)) if which == 0 else (f(q, a) - f(q, b_))) / (2 * eps)
            assert np.allclose(num, grad, atol=1e-7), which


def test_dropout_matches_loops_and_rate():
    B, Sq, Sk, nh, dh = 2, 4, 3, 2, 4
    q = rng.normal(size=(B * Sq, nh * dh)); kv = rng.normal(size=(B * Sk, 2 * nh * dh))
    keep = [D.keep_cross_attention(9, 0, 2, b, nh, Sq, Sk, 0.25) for b in range(B)]
    o, lse = O.cross_attention_fwd(q, kv, B, Sq, Sk, nh, lambda b: keep[b], D.scale(0.25))
    o2, lse2 = _brute(q, kv, B, Sq, Sk, nh, keep, D.scale(0.25))
    assert np.allclose(o, o2, atol=1e-12) and np.allclose(lse, lse2, atol=1e-12)
    # the mask: right rate, its own site (differs from the self-attention mask of the same shape), and
    # position query*Sk + key (a [Sq, Sk] mask is the row-major reshape of the flat index range)
    big = D.keep_cross_attention(9, 0, 2, 0, 2, 300, 200, 0.25)
    assert abs(big.mean() - 0.75) < 0.01
    sq = D.keep_cross_attention(9, 0, 2, 0, 2, 64, 64, 0.25)
    assert (sq != D.keep_attention(9, 0, 2, 0, 2, 64, 0.25)).mean() > 0.3
    k0, k1 = D.unit_keys(D.site_base(9, 0, 2, D.SITE_CROSS), 1)
    with np.errstate(over="ignore"):
        flat = D.bits(np.arange(300 * 200, dtype=np.uint32), k0, k1) >= np.uint32(D.threshold(0.25))
    assert np.array_equal(big[1], flat.reshape(300, 200))


def test_matches_torch_autograd():
    torch = pytest.importorskip("torch")
    B, Sq, Sk, nh, dh = 2, 5, 7, 3, 4
    H = nh * dh
    q = rng.normal(size=(B * Sq, H)); kv = rng.normal(size=(B * Sk, 2 * H)); do = rng.normal(size=(B * Sq, H))
    tq = torch.tensor(q, requires_grad=True); tkv = torch.tensor(kv, requires_grad=True)
    qh = tq.reshape(B, Sq, nh, dh).permute(0, 2, 1, 3)
    kh = tkv[:, :H].reshape(B, Sk, nh, dh).permute(0, 2, 1, 3)
    vh = tkv[:, H:].reshape(B, Sk, nh, dh).permute(0, 2, 1, 3)
    to = torch.nn.functional.scaled_dot_product_attention(qh, kh, vh).permute(0, 2, 1, 3).reshape(B * Sq, H)
    to.backward(torch.tensor(do))
    o, _ = O.cross_attention_fwd(q, kv, B, Sq, Sk, nh)
    dq, dkv = O.cross_attention_bwd(do, q, kv, B, Sq, Sk, nh)
    assert np.allclose(o, to.detach().numpy(), atol=1e-12)
    assert np.allclose(dq, tq.grad.numpy(), atol=1e-12) and np.allclose(dkv, tkv.grad.numpy(), atol=1e-12)
