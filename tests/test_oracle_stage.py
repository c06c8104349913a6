"""Pins for the oracle's stage step: finite differences, an independent autograd
evaluation, closed-form special cases, structural invariants, plan invariance."""
import itertools

import numpy as np
import pytest

import synthetic as syn
from oracle import stage as O


def tiny(style, causal, gelu, L=2, H=16, nh=2, F=32, S=5, B=2):
    cfg = syn.StageConfig(L, H, nh, F, S, B, style, causal, gelu, "f32")
    st = O.Stage(L, H, nh, F, S, B, style, causal, gelu, cfg.ln_eps)
    w = syn.make_weights(cfg, seed=0, sigma=0.3)
    w = [{k: v.astype(np.float64) for k, v in d.items()} for d in w]
    x, dy = syn.make_activations(cfg)
    return cfg, st, w, x.astype(np.float64), dy.astype(np.float64)


VARIANTS = list(itertools.product(["pre", "post"], [False, True], ["erf", "tanh"]))


@pytest.mark.parametrize("style,causal,gelu", VARIANTS)
def test_finite_differences(style, causal, gelu):
    """dL/dtheta along random directions, L = <Y, dY>, central differences."""
    cfg, st, w, x, dy = tiny(style, causal, gelu)
    y, dx, grads = O.stage_step(st, w, x, dy)
    rng = np.random.default_rng(7)
    h = 1e-6

    def loss(ws, xx):
        return float((O.stage_forward(st, ws, xx) * dy).sum())

    u = rng.normal(size=x.shape)
    fd = (loss(w, x + h * u) - loss(w, x - h * u)) / (2 * h)
    assert np.isclose(fd, (dx * u).sum(), rtol=2e-6, atol=1e-7)
    for l in range(cfg.n_layers):
        for name in syn.WEIGHT_NAMES:
            u = rng.normal(size=w[l][name].shape)
            wp = [dict(d) for d in w]; wm = [dict(d) for d in w]
            wp[l][name] = w[l][name] + h * u
            wm[l][name] = w[l][name] - h * u
            fd = (loss(wp, x) - loss(wm, x)) / (2 * h)
            an = float((grads[l][name] * u).sum())
            assert np.isclose(fd, an, rtol=2e-6, atol=1e-7), (l, name, fd, an)


@pytest.mark.parametrize("style,causal,gelu", VARIANTS)
def test_matches_torch_autograd(style, causal, gelu):
    """A second evaluation of the same stage by torch's CPU autograd (float64)."""
    torch = pytest.importorskip("torch")
    Fn = torch.nn.functional
    cfg, st, w, x, dy = tiny(style, causal, gelu)
    H, nh, S, B = cfg.hidden, cfg.n_heads, cfg.seq, cfg.micro_batch
    dh = H // nh
    tw = [{k: torch.tensor(v, requires_grad=True) for k, v in d.items()} for d in w]
    tx = torch.tensor(x, requires_grad=True)

    def attn(qkv):
        q, k, v = (qkv[:, i * H:(i + 1) * H].reshape(B, S, nh, dh).permute(0, 2, 1, 3) for i in range(3))
        o = Fn.scaled_dot_product_attention(q, k, v, is_causal=causal)
        return o.permute(0, 2, 1, 3).reshape(B * S, H)

    def act(v):
        return Fn.gelu(v, approximate="none" if gelu == "erf" else "tanh")

    h = tx
    for p in tw:
        if style == "pre":
            a = Fn.layer_norm(h, (H,), p["ln1_g"], p["ln1_b"], cfg.ln_eps)
            m = h + attn(a @ p["w_qkv"] + p["b_qkv"]) @ p["w_o"] + p["b_o"]
            c = Fn.layer_norm(m, (H,), p["ln2_g"], p["ln2_b"], cfg.ln_eps)
            h = m + act(c @ p["w_fc1"] + p["b_fc1"]) @ p["w_fc2"] + p["b_fc2"]
        else:
            r1 = h + attn(h @ p["w_qkv"] + p["b_qkv"]) @ p["w_o"] + p["b_o"]
            m = Fn.layer_norm(r1, (H,), p["ln1_g"], p["ln1_b"], cfg.ln_eps)
            r2 = m + act(m @ p["w_fc1"] + p["b_fc1"]) @ p["w_fc2"] + p["b_fc2"]
            h = Fn.layer_norm(r2, (H,), p["ln2_g"], p["ln2_b"], cfg.ln_eps)
    h.backward(torch.tensor(dy))
    y, dx, grads = O.stage_step(st, w, x, dy)
    assert np.allclose(y, h.detach().numpy(), atol=1e-11)
    assert np.allclose(dx, tx.grad.numpy(), atol=1e-10)
    for l in range(cfg.n_layers):
        for name in syn.WEIGHT_NAMES:
            assert np.allclose(grads[l][name], tw[l][name].grad.numpy(), atol=1e-10), (l, name)


def test_identity_stage_pre_ln():
    """Pre-LN with W_o = b_o = W_2 = b_2 = 0 is the identity: Y = X, dX = dY,
    and dW_o = ATTN_OUT^T dY."""
    cfg, st, w, x, dy = tiny("pre", True, "erf", L=1)
    for n in ("w_o", "b_o", "w_fc2", "b_fc2"):
        w[0][n] = np.zeros_like(w[0][n])
    y, dx, g = O.stage_step(st, w, x, dy)
    assert np.array_equal(y, x) and np.allclose(dx, dy, atol=1e-14)
    _, s = st.layer_fwd(x, w[0])
    o = s["ATTN_OUT"]
    ref = np.zeros_like(w[0]["w_o"])
    for t in range(x.shape[0]):
        for k in range(cfg.hidden):
            for n in range(cfg.hidden):
                ref[k, n] += o[t, k] * dy[t, n]
    assert np.allclose(g[0]["w_o"], ref, atol=1e-12)
    assert np.allclose(g[0]["b_fc2"], dy.sum(axis=0))


@pytest.mark.parametrize("style", ["pre", "post"])
def test_batch_independence(style):
    cfg, st, w, x, dy = tiny(style, False, "erf")
    S, T = cfg.seq, cfg.tokens
    y, dx, g = O.stage_step(st, w, x, dy)
    # perturb sample 1 only: sample 0 results unchanged
    x2 = x.copy(); x2[S:] += 1.0
    y2, dx2, _ = O.stage_step(st, w, x2, dy)
    assert np.array_equal(y[:S], y2[:S]) and np.array_equal(dx[:S], dx2[:S])
    # weight gradients add over samples
    st1 = O.Stage(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, S, 1, style, False, "erf", cfg.ln_eps)
    _, _, ga = O.stage_step(st1, w, x[:S], dy[:S])
    _, _, gb = O.stage_step(st1, w, x[S:], dy[S:])
    for l in range(cfg.n_layers):
        for n in syn.WEIGHT_NAMES:
            assert np.allclose(g[l][n], ga[l][n] + gb[l][n], atol=1e-11)


def test_causal_prefix_property():
    cfg, st, w, x, dy = tiny("pre", True, "erf", B=1, S=6)
    y = O.stage_forward(st, w, x)
    x2 = x.copy(); x2[4:] = 3.0 - x2[4:]
    y2 = O.stage_forward(st, w, x2)
    assert np.array_equal(y[:4], y2[:4]) and not np.allclose(y[4:], y2[4:])
    # without the mask the prefix does change
    st_nc = O.Stage(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, 6, 1, "pre", False, "erf", cfg.ln_eps)
    assert not np.allclose(O.stage_forward(st_nc, w, x)[:4], O.stage_forward(st_nc, w, x2)[:4])


def test_head_permutation_invariance():
    cfg, st, w, x, dy = tiny("post", False, "erf", L=1)
    H, nh = cfg.hidden, cfg.n_heads
    dh = H // nh
    perm = np.concatenate([np.arange(dh) + dh * h for h in reversed(range(nh))])
    w2 = [dict(w[0])]
    cols = np.concatenate([perm, H + perm, 2 * H + perm])
    w2[0]["w_qkv"] = w[0]["w_qkv"][:, cols]; w2[0]["b_qkv"] = w[0]["b_qkv"][cols]
    w2[0]["w_o"] = w[0]["w_o"][perm, :]
    assert np.allclose(O.stage_forward(st, w, x), O.stage_forward(st, w2, x), atol=1e-12)


@pytest.mark.parametrize("style", ["pre", "post"])
def test_plan_invariance(style):
    cfg, st, w, x, dy = tiny(style, style == "pre", "erf", L=3)
    y, dx, g = O.stage_step(st, w, x, dy)
    plans = [syn.plan_keep_all(cfg), syn.plan_all_recompute(cfg), syn.plan_all_swap(cfg),
             syn.plan_uniform(cfg, syn.RECOMPUTE), syn.plan_recompute_attention(cfg),
             syn.plan_swap_ffn_recompute_norm_gelu(cfg)]
    plans += [syn.plan_seeded(cfg, s) for s in range(100)]
    for p in plans:
        y2, dx2, g2, c = O.stage_step_under_plan(st, w, x, dy, p)
        assert np.array_equal(y, y2) and np.array_equal(dx, dx2)
        for l in range(cfg.n_layers):
            for n in syn.WEIGHT_NAMES:
                assert np.array_equal(g[l][n], g2[l][n])
        pm = p.reshape(cfg.n_layers, -1)
        assert c["swapped_out"] == c["swapped_in"] == int((pm == syn.SWAP).sum())
        assert (c["replayed"] > 0) == bool((pm == syn.RECOMPUTE).any())


def test_float32_close_to_float64():
    cfg, st, w, x, dy = tiny("pre", True, "erf", L=2, H=32, nh=2, F=64, S=16, B=2)
    y, dx, g = O.stage_step(st, w, x, dy)
    y32, dx32, g32 = O.stage_step(st, w, x, dy, dtype=np.float32)
    assert y32.dtype == np.float32
    assert O.max_rel_err(y32, y) < 1e-5 and O.max_rel_err(dx32, dx) < 1e-5
    for l in range(2):
        for n in syn.WEIGHT_NAMES:
            assert O.max_rel_err(g32[l][n], g[l][n]) < 1e-5


def test_inputs_module():
    # splitmix64 reference values for seed 0 (first outputs of the published generator)
    z = syn.splitmix64(0, np.arange(3, dtype=np.uint64))
    assert [int(v) for v in z] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    n = syn.normal(3, 0, 200000)
    assert abs(n.mean()) < 0.01 and abs(n.std() - 1) < 0.01
    assert np.array_equal(syn.normal(3, 100, 50), n[100:150])
    # bf16 rounding: ties to even, exact values unchanged
    a = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7, 3.14159], dtype=np.float32)
    r = syn.round_to_bf16(a)
    assert list(r[:4]) == [1.0, 1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7]
    assert abs(r[4] - 3.140625) < 1e-9
    torch = pytest.importorskip("torch")
    big = syn.normal(5, 0, 10000).astype(np.float32)
    assert np.array_equal(syn.round_to_bf16(big), torch.tensor(big).to(torch.bfloat16).float().numpy())
    cfg = syn.CONFIGS["C5"]
    p = syn.plan_seeded(cfg, 7).reshape(cfg.n_layers, -1)
    assert p[0, 0] == syn.KEEP and np.all(p[:, syn.SLOT["RES2"]] == syn.KEEP)
    assert set(np.unique(p)) == {0, 1, 2}
    assert abs(syn.CONFIGS["C2"].model_flops() - 2.010e12) / 2.010e12 < 2e-3
    assert abs(syn.CONFIGS["C3"].model_flops() - 6.362e12) / 6.362e12 < 2e-3


@pytest.mark.parametrize("style", ["pre", "post"])
def test_relu_with_decisions_given_from_outside(style):
    """The test-only switch that lets a ReLU stage use decisions x > 0 taken elsewhere: with the stage's own
    decisions nothing changes (bit for bit); with some of them flipped the stage computes x -> x [given], a smooth
    function of its inputs, and its gradients are the derivatives of exactly that function (central differences)."""
    cfg, st, w, x, dy = tiny(style, False, "relu")
    y0, dx0, g0 = O.stage_step(st, w, x, dy)
    own, h_in = [], x
    for l in range(cfg.n_layers):
        h_in, saved = st.layer_fwd(h_in, w[l], l)
        own.append(saved["FC1_OUT"] > 0)
    st.relu_decisions = own
    y1, dx1, g1 = O.stage_step(st, w, x, dy)
    assert np.array_equal(y0, y1) and np.array_equal(dx0, dx1)
    assert all(np.array_equal(g0[l][n], g1[l][n]) for l in range(cfg.n_layers) for n in syn.WEIGHT_NAMES)
    rng = np.random.default_rng(3)
    flipped = [d ^ (rng.random(d.shape) < 0.1) for d in own]
    assert any((a != b).any() for a, b in zip(own, flipped))
    st.relu_decisions = flipped
    y2, dx2, g2 = O.stage_step(st, w, x, dy)
    assert not np.array_equal(y0, y2)
    hh = 1e-6

    def loss(ws, xx):
        return float((O.stage_forward(st, ws, xx) * dy).sum())

    u = rng.normal(size=x.shape)
    fd = (loss(w, x + hh * u) - loss(w, x - hh * u)) / (2 * hh)
    assert np.isclose(fd, (dx2 * u).sum(), rtol=2e-6, atol=1e-7)
    for name in ("w_fc1", "b_fc1", "w_fc2", "ln1_g", "w_qkv"):
        u = rng.normal(size=w[0][name].shape)
        wp = [dict(d) for d in w]; wm = [dict(d) for d in w]
        wp[0][name] = w[0][name] + hh * u
        wm[0][name] = w[0][name] - hh * u
        fd = (loss(wp, x) - loss(wm, x)) / (2 * hh)
        assert np.isclose(fd, float((g2[0][name] * u).sum()), rtol=2e-6, atol=1e-7), name
