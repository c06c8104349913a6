"""Pins for the oracle's multi-micro-batch schedule (one stage of a one-forward-one-backward
pipeline, Section 1): what the mathematics fixes, not the oracle's own formula."""
import numpy as np
import pytest

import synthetic as syn
from oracle import stage as O


def micro_batches(n, style="pre", causal=True, L=2, H=16, nh=2, F=32, S=5, B=2):
    cfg = syn.StageConfig(L, H, nh, F, S, B, style, causal, "erf", "f32")
    st = O.Stage(L, H, nh, F, S, B, style, causal, "erf", cfg.ln_eps)
    w = [{k: v.astype(np.float64) for k, v in d.items()} for d in syn.make_weights(cfg, seed=0, sigma=0.3)]
    xs, dys = [], []
    for m in range(n):
        x, dy = syn.make_activations(cfg, seed_x=11 + 2 * m, seed_dy=12 + 2 * m)
        xs.append(x.astype(np.float64)); dys.append(dy.astype(np.float64))
    return cfg, st, w, xs, dys


@pytest.mark.parametrize("n,inflight", [(1, 1), (4, 1), (4, 2), (5, 3), (3, 4), (6, 6)])
def test_order_is_a_valid_1f1b_schedule(n, inflight):
    order = O.one_f_one_b(n, inflight)
    assert sorted(order) == sorted([("F", m) for m in range(n)] + [("B", m) for m in range(n)])
    held, most, last_b = set(), 0, -1
    for i, (kind, m) in enumerate(order):
        if kind == "F":
            held.add(m)
        else:
            assert m in held and m == last_b + 1      # backwards in feeding order, after their forward
            held.remove(m); last_b = m
        most = max(most, len(held))
        assert len(held) <= inflight
    assert most == min(inflight, n)
    # steady state alternates: after the fill, no two forwards in a row
    fill = min(inflight, n)
    kinds = [k for k, _ in order[fill:]]
    assert all(not (a == "F" and b == "F") for a, b in zip(kinds, kinds[1:]))


@pytest.mark.parametrize("style,causal", [("pre", True), ("post", False)])
def test_summed_gradients_equal_the_concatenated_batch(style, causal):
    """Sequences do not interact inside a stage, and a weight gradient is a sum over tokens:
    n micro-batches of B sequences give the gradients of one batch of n*B sequences."""
    n = 3
    cfg, st, w, xs, dys = micro_batches(n, style, causal)
    ys, dxs, g, most = O.stage_schedule(st, w, xs, dys, O.one_f_one_b(n, 2))
    assert most == 2
    big = O.Stage(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, n * cfg.micro_batch, style, causal,
                  "erf", cfg.ln_eps)
    yb, dxb, gb = O.stage_step(big, w, np.concatenate(xs, 0), np.concatenate(dys, 0))
    np.testing.assert_allclose(np.concatenate(ys, 0), yb, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(np.concatenate(dxs, 0), dxb, rtol=1e-12, atol=1e-13)
    for l in range(cfg.n_layers):
        for k in syn.WEIGHT_NAMES:
            np.testing.assert_allclose(g[l][k], gb[l][k], rtol=1e-10, atol=1e-12)


def test_every_event_order_gives_the_same_results():
    n = 4
    cfg, st, w, xs, dys = micro_batches(n)
    ref = O.stage_schedule(st, w, xs, dys, O.one_f_one_b(n, 1))
    gpipe = [("F", m) for m in range(n)] + [("B", m) for m in reversed(range(n))]
    for order in (O.one_f_one_b(n, 2), O.one_f_one_b(n, 4), gpipe):
        got = O.stage_schedule(st, w, xs, dys, order)
        for a, b in zip(got[0] + got[1], ref[0] + ref[1]):
            assert np.array_equal(a, b)                      # per-micro-batch results do not depend on the order
        for l in range(cfg.n_layers):
            for k in syn.WEIGHT_NAMES:
                np.testing.assert_allclose(got[2][l][k], ref[2][l][k], rtol=1e-12, atol=1e-13)


def test_single_micro_batch_is_the_plain_step():
    cfg, st, w, xs, dys = micro_batches(1)
    ys, dxs, g, most = O.stage_schedule(st, w, xs, dys, O.one_f_one_b(1, 1))
    y, dx, gr = O.stage_step(st, w, xs[0], dys[0])
    assert most == 1 and np.array_equal(ys[0], y) and np.array_equal(dxs[0], dx)
    assert all(np.array_equal(g[l][k], gr[l][k]) for l in range(cfg.n_layers) for k in syn.WEIGHT_NAMES)


def test_a_schedule_with_a_missing_backward_is_rejected():
    cfg, st, w, xs, dys = micro_batches(2)
    with pytest.raises(AssertionError):
        O.stage_schedule(st, w, xs, dys, [("F", 0), ("F", 1), ("B", 0)])


# ---------------------------------------------------------------- parameter versions (asynchronous schedule)
def two_versions(n=2):
    cfg, st, w0, xs, dys = micro_batches(n)
    w1 = [{k: v.astype(np.float64) for k, v in d.items()} for d in syn.make_weights(cfg, seed=5, sigma=0.3)]
    return cfg, st, [w0, w1], xs, dys


def test_backward_differentiates_the_version_its_forward_used():
    """Micro-batch 0 is fed under version 0, version 1 becomes current before its backward:
    dX must be the gradient of <Y, dY> with version 0's parameters (central differences), and
    is measurably not the gradient under version 1."""
    cfg, st, vs, xs, dys = two_versions()
    order = [("W", 0), ("F", 0), ("W", 1), ("F", 1), ("B", 0), ("B", 1)]
    ys, dxs, grads, used, most = O.stage_schedule_async(st, vs, xs, dys, order)
    assert used == [0, 1] and most == 2
    rng = np.random.default_rng(3)
    h = 1e-6
    for m in (0, 1):
        u = rng.normal(size=xs[m].shape)
        def loss(ws, xx):
            return float((O.stage_forward(st, ws, xx) * dys[m]).sum())
        fd = {v: (loss(vs[v], xs[m] + h * u) - loss(vs[v], xs[m] - h * u)) / (2 * h) for v in (0, 1)}
        got = float((dxs[m] * u).sum())
        assert np.isclose(got, fd[used[m]], rtol=2e-6, atol=1e-7)
        assert not np.isclose(got, fd[1 - used[m]], rtol=1e-3)
        # and a parameter gradient, along a random direction of one matrix
        d = rng.normal(size=vs[0][0]["w_fc1"].shape)
        def shifted(ws, t):
            out = [dict(layer) for layer in ws]
            out[0]["w_fc1"] = out[0]["w_fc1"] + t * d
            return out
        fdw = (loss(shifted(vs[used[m]], h), xs[m]) - loss(shifted(vs[used[m]], -h), xs[m])) / (2 * h)
        assert np.isclose(float((grads[m][0]["w_fc1"] * d).sum()), fdw, rtol=2e-6, atol=1e-7)


def test_without_updates_in_flight_one_version_suffices():
    cfg, st, vs, xs, dys = two_versions()
    order = [("W", 0), ("F", 0), ("B", 0), ("W", 1), ("F", 1), ("B", 1)]
    *_, used, most = O.stage_schedule_async(st, vs, xs, dys, order)
    assert used == [0, 1] and most == 1


@pytest.mark.parametrize("inflight", [1, 2, 3])
def test_an_update_after_every_backward_needs_one_version_per_micro_batch_in_flight(inflight):
    """Section 1: a stage with k micro-batches in flight keeps k parameter versions."""
    n = 6
    cfg, st, w, xs, dys = micro_batches(n, L=1, S=3, B=1)
    versions = [w] * (n + 1)           # the values do not matter for the count
    order, v = [("W", 0)], 0
    for kind, m in O.one_f_one_b(n, inflight):
        order.append((kind, m))
        if kind == "B":
            v += 1
            order.append(("W", v))
    *_, used, most = O.stage_schedule_async(st, versions, xs, dys, order)
    assert most == inflight
    assert used == [max(0, m - inflight + 1) for m in range(n)]
