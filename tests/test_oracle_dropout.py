"""Pins for the dropout oracle: properties of the counter-based mask generator that any sound
generator must have, and the stage step with masks against central differences and against
attention written out element by element."""
import math

import numpy as np
import pytest

import synthetic as syn
from oracle import dropout as D
from oracle import stage as O


# ---------------------------------------------------------------- the generator
def test_mixer_is_injective_and_avalanches():
    x = np.arange(1 << 20, dtype=np.uint32)
    y = D.mix(x)
    assert len(np.unique(y)) == len(x)                       # a bijection never collides
    # flipping one input bit flips about half of the output bits, for every input bit
    for bit in range(32):
        d = y ^ D.mix(x ^ np.uint32(1 << bit))
        flipped = np.unpackbits(d.view(np.uint8)).mean() * 32
        assert 14.5 < flipped < 17.5, (bit, flipped)


def test_mixer_inverts():
    """Each step of the mixer has a closed-form inverse (xorshift undone by repeated shifts,
    odd multiplier by its inverse mod 2^32): applying them in reverse order returns the input,
    which fixes the constants and the shift amounts, not only some bijection."""
    inv1, inv2 = pow(D.M1, -1, 1 << 32), pow(D.M2, -1, 1 << 32)
    x = np.arange(12345, 12345 + 4096, dtype=np.uint32) * np.uint32(2654435761)
    y = D.mix(x).astype(np.uint64)
    y ^= y >> 16
    y = (y * inv2) & 0xFFFFFFFF
    y ^= (y >> 15) ^ (y >> 30)
    y = (y * inv1) & 0xFFFFFFFF
    y ^= y >> 16
    assert np.array_equal(y.astype(np.uint32), x)


@pytest.mark.parametrize("p", [0.1, 0.25, 0.5])
def test_keep_rate(p):
    n = 1 << 20
    for unit in (0, 1, 77):
        k0, k1 = D.unit_keys(D.site_base(3, 5, 2, 1), unit)
        keep = D.bits(np.arange(n, dtype=np.uint32), k0, k1) >= np.uint32(D.threshold(p))
        sigma = math.sqrt(p * (1 - p) / n)
        assert abs(keep.mean() - (1 - p)) < 4.5 * sigma


def _independent(a, b, p):
    """two keep masks with rate 1-p: the joint rate of (drop, drop) is p^2 within 4.5 sigma"""
    n = a.size
    both = (~a & ~b).mean()
    return abs(both - p * p) < 4.5 * math.sqrt(p * p * (1 - p * p) / n)


def test_masks_are_pairwise_independent_across_everything_that_distinguishes_them():
    p, T, H = 0.3, 512, 512
    ref = D.keep_hidden(7, 11, 3, D.SITE_PROJ, T, H, p)
    assert _independent(ref[:, :-1], ref[:, 1:], p)          # neighbours in a row
    assert _independent(ref[:-1], ref[1:], p)                # neighbours in a column
    others = [D.keep_hidden(8, 11, 3, D.SITE_PROJ, T, H, p), D.keep_hidden(7 + (1 << 32), 11, 3, D.SITE_PROJ, T, H, p),
              D.keep_hidden(7, 12, 3, D.SITE_PROJ, T, H, p), D.keep_hidden(7, 11 + (1 << 32), 3, D.SITE_PROJ, T, H, p),
              D.keep_hidden(7, 11, 4, D.SITE_PROJ, T, H, p), D.keep_hidden(7, 11, 3, D.SITE_FC2, T, H, p)]
    for o in others:
        assert not np.array_equal(o, ref) and _independent(ref, o, p)
    assert np.array_equal(ref, D.keep_hidden(7, 11, 3, D.SITE_PROJ, T, H, p))     # a pure function
    a = D.keep_attention(7, 11, 3, 1, 4, 128, p)
    assert _independent(a[0], a[1], p) and _independent(a[0], a[0].T, p)
    assert _independent(a[2], D.keep_attention(7, 11, 3, 0, 4, 128, p)[2], p)      # other sample, same head
    assert _independent(a[:, :, :-1], a[:, :, 1:], p) and _independent(a[:, :-1], a[:, 1:], p)


def test_threshold_and_scale():
    assert D.threshold(0.0) == 0 and D.threshold(0.5) == 1 << 31
    assert D.threshold(0.1) == int(math.floor(float(np.float32(0.1)) * 2 ** 32))
    assert D.keep_hidden(1, 2, 0, 1, 64, 64, 0.0).all()
    assert math.isclose(D.scale(0.25), 4 / 3)


# ---------------------------------------------------------------- the stage step with masks
def tiny(style, causal, p_attn, p_hidden, L=2, H=16, nh=2, F=32, S=6, B=2):
    cfg = syn.StageConfig(L, H, nh, F, S, B, style, causal, "erf", "f32")
    st = O.Stage(L, H, nh, F, S, B, style, causal, "erf", cfg.ln_eps, p_attn=p_attn, p_hidden=p_hidden)
    st.set_rng(1234, 5)
    w = [{k: v.astype(np.float64) for k, v in d.items()} for d in syn.make_weights(cfg, seed=0, sigma=0.3)]
    x, dy = syn.make_activations(cfg)
    return cfg, st, w, x.astype(np.float64), dy.astype(np.float64)


@pytest.mark.parametrize("style,causal", [("pre", True), ("post", False)])
@pytest.mark.parametrize("p_attn,p_hidden", [(0.3, 0.0), (0.0, 0.3), (0.2, 0.4)])
def test_finite_differences_with_masks(style, causal, p_attn, p_hidden):
    """With the masks fixed the step is differentiable; every gradient along random directions."""
    cfg, st, w, x, dy = tiny(style, causal, p_attn, p_hidden)
    y, dx, grads = O.stage_step(st, w, x, dy)
    rng = np.random.default_rng(7)
    h = 1e-6

    def loss(ws, xx):
        return float((O.stage_forward(st, ws, xx) * dy).sum())

    u = rng.normal(size=x.shape)
    assert np.isclose((loss(w, x + h * u) - loss(w, x - h * u)) / (2 * h), (dx * u).sum(), rtol=2e-6, atol=1e-7)
    for l in range(cfg.n_layers):
        for name in syn.WEIGHT_NAMES:
            u = rng.normal(size=w[l][name].shape)
            wp = [dict(d) for d in w]; wm = [dict(d) for d in w]
            wp[l][name] = w[l][name] + h * u; wm[l][name] = w[l][name] - h * u
            fd = (loss(wp, x) - loss(wm, x)) / (2 * h)
            assert np.isclose(fd, (grads[l][name] * u).sum(), rtol=5e-6, atol=1e-7), (l, name)


def test_zero_rate_is_the_plain_step_and_the_mask_matters():
    cfg, st, w, x, dy = tiny("pre", True, 0.0, 0.0)
    plain = O.stage_step(st, w, x, dy)
    st.set_rng(99, 1)
    again = O.stage_step(st, w, x, dy)
    assert np.array_equal(plain[0], again[0]) and np.array_equal(plain[1], again[1])
    cfg, sd, w, x, dy = tiny("pre", True, 0.2, 0.2)
    a = O.stage_step(sd, w, x, dy)
    sd.set_rng(1234, 6)                     # the next micro-batch draws other masks
    b = O.stage_step(sd, w, x, dy)
    sd.set_rng(1234, 5)
    c = O.stage_step(sd, w, x, dy)
    assert not np.allclose(a[0], plain[0]) and not np.allclose(a[0], b[0]) and np.array_equal(a[0], c[0])


def test_attention_with_dropout_element_by_element():
    B, S, nh, dh = 2, 5, 2, 4
    H = nh * dh
    rng = np.random.default_rng(0)
    qkv = rng.normal(size=(B * S, 3 * H))
    p = 0.4
    keep = lambda b: D.keep_attention(9, 0, 1, b, nh, S, p)
    out, lse = O.attention_fwd(qkv, B, S, nh, True, keep, D.scale(p))
    plain, lse0 = O.attention_fwd(qkv, B, S, nh, True)
    assert np.array_equal(lse, lse0)
    for b in range(B):
        kb = keep(b)
        for h in range(nh):
            for i in range(S):
                q = qkv[b * S + i, h * dh:(h + 1) * dh]
                logits = [q @ qkv[b * S + j, H + h * dh:H + (h + 1) * dh] / math.sqrt(dh) for j in range(i + 1)]
                z = sum(math.exp(a) for a in logits)
                o = np.zeros(dh)
                for j in range(i + 1):
                    if kb[h, i, j]:
                        o += math.exp(logits[j]) / z / (1 - float(np.float32(p))) * qkv[b * S + j, 2 * H + h * dh:2 * H + (h + 1) * dh]
                np.testing.assert_allclose(out[b * S + i, h * dh:(h + 1) * dh], o, rtol=1e-12, atol=1e-13)


def test_dropout_is_unbiased_over_micro_batches():
    """The mean over many masks of a dropped hidden state is the state itself."""
    T, H, p = 8, 16, 0.3
    x = np.random.default_rng(1).normal(size=(T, H))
    acc = np.zeros_like(x)
    n = 4000
    for mb in range(n):
        acc += x * D.keep_hidden(5, mb, 0, D.SITE_FC2, T, H, p) * D.scale(p)
    err = np.abs(acc / n - x) / np.abs(x)
    # per-element standard error is |x| sqrt(p/(1-p)/n) = 1.04 % of |x|
    assert err.max() < 5 * math.sqrt(p / (1 - p) / n)


def test_plans_do_not_change_the_numbers_with_dropout():
    cfg, st, w, x, dy = tiny("pre", True, 0.2, 0.3)
    ref = O.stage_step(st, w, x, dy)
    for plan in (syn.plan_all_recompute(cfg), syn.plan_all_swap(cfg), syn.plan_seeded(cfg, 4)):
        got = O.stage_step_under_plan(st, w, x, dy, plan)
        assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
        assert all(np.array_equal(got[2][l][k], ref[2][l][k]) for l in range(cfg.n_layers) for k in syn.WEIGHT_NAMES)
