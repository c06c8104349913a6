"""Pins for the oracle's operators: closed forms, identities, brute force and
library special cases.  None of these re-types the oracle's own formula."""
import math

import numpy as np
import pytest

from oracle import stage as O

rng = np.random.default_rng(1234)


# ---------------------------------------------------------------- linear
def test_linear_bwd_triple_loops():
    x = rng.normal(size=(5, 4)); w = rng.normal(size=(4, 3)); dy = rng.normal(size=(5, 3))
    dx, dw, db = O.linear_bwd(dy, x, w)
    dx2 = np.zeros_like(x); dw2 = np.zeros_like(w); db2 = np.zeros(3)
    for t in range(5):
        for n in range(3):
            db2[n] += dy[t, n]
            for k in range(4):
                dx2[t, k] += dy[t, n] * w[k, n]
                dw2[k, n] += x[t, k] * dy[t, n]
    assert np.allclose(dx, dx2) and np.allclose(dw, dw2) and np.allclose(db, db2)
    # layout: W is [in, out]
    y = O.linear_fwd(x, w, np.arange(3.0))
    assert y.shape == (5, 3)
    assert np.isclose(y[2, 1], sum(x[2, k] * w[k, 1] for k in range(4)) + 1.0)


# ---------------------------------------------------------------- LayerNorm
def test_layernorm_identities():
    H = 48
    x = rng.normal(size=(7, H)) * 3 + 1.5
    one, zero = np.ones(H), np.zeros(H)
    eps = 1e-5
    y, mu, r = O.layernorm_fwd(x, one, zero, eps)
    assert np.allclose(y.sum(axis=1), 0, atol=1e-12)
    var = x.var(axis=1)                       # numpy's biased variance
    assert np.allclose((y * y).sum(axis=1), H * var / (var + eps), rtol=1e-12)
    assert np.allclose(mu, x.mean(axis=1)) and np.allclose(r, 1 / np.sqrt(var + eps))
    # invariance to positive scaling and shift (eps makes it approximate)
    y2, _, _ = O.layernorm_fwd(2.5 * x + 7.0, one, zero, eps)
    assert np.allclose(y, y2, atol=1e-5)
    # affine part
    g, b = rng.normal(size=H), rng.normal(size=H)
    y3, _, _ = O.layernorm_fwd(x, g, b, eps)
    assert np.allclose(y3, y * g + b)


def test_layernorm_bwd_orthogonality_and_sums():
    H = 32
    x = rng.normal(size=(6, H)); dy = rng.normal(size=(6, H)); g = rng.normal(size=H)
    # eps -> 0 so that sum(xhat^2) = H and the second orthogonality is exact
    y, mu, r = O.layernorm_fwd(x, np.ones(H), np.zeros(H), 1e-14)
    dx, dg, db = O.layernorm_bwd(dy, x, mu, r, g)
    assert np.allclose(dx.sum(axis=1), 0, atol=1e-12)          # dx orthogonal to 1
    assert np.allclose((dx * y).sum(axis=1), 0, atol=1e-10)    # dx orthogonal to xhat
    assert np.allclose(db, dy.sum(axis=0))
    assert np.allclose(dg, (dy * y).sum(axis=0))


def test_layernorm_matches_torch():
    torch = pytest.importorskip("torch")
    H = 24
    x = rng.normal(size=(5, H)); g = rng.normal(size=H); b = rng.normal(size=H); dy = rng.normal(size=(5, H))
    tx = torch.tensor(x, requires_grad=True); tg = torch.tensor(g, requires_grad=True)
    tb = torch.tensor(b, requires_grad=True)
    ty = torch.nn.functional.layer_norm(tx, (H,), tg, tb, 1e-5)
    ty.backward(torch.tensor(dy))
    y, mu, r = O.layernorm_fwd(x, g, b, 1e-5)
    dx, dg, db = O.layernorm_bwd(dy, x, mu, r, g)
    assert np.allclose(y, ty.detach().numpy(), atol=1e-12)
    assert np.allclose(dx, tx.grad.numpy(), atol=1e-12)
    assert np.allclose(dg, tg.grad.numpy(), atol=1e-12)
    assert np.allclose(db, tb.grad.numpy(), atol=1e-12)


# ---------------------------------------------------------------- GELU
@pytest.mark.parametrize("kind", ["erf", "tanh"])
def test_gelu_identities(kind):
    x = np.linspace(-6, 6, 241)
    g = O.gelu_fwd(x, kind)
    assert O.gelu_fwd(np.zeros(1), kind)[0] == 0.0
    assert np.isclose(O.gelu_grad(np.zeros(1), kind)[0], 0.5)
    assert np.allclose(g - O.gelu_fwd(-x, kind), x, atol=1e-12)   # g(x) - g(-x) = x
    big = np.array([12.0, 30.0])
    assert np.allclose(O.gelu_fwd(big, kind), big) and np.allclose(O.gelu_fwd(-big, kind), 0, atol=1e-12)
    assert np.allclose(O.gelu_grad(big, kind), 1) and np.allclose(O.gelu_grad(-big, kind), 0, atol=1e-12)
    # derivative against central differences
    h = 1e-6
    fd = (O.gelu_fwd(x + h, kind) - O.gelu_fwd(x - h, kind)) / (2 * h)
    assert np.allclose(O.gelu_grad(x, kind), fd, atol=1e-8)


def test_relu_by_its_definition():
    x = np.array([-3.0, -1e-9, 0.0, 1e-9, 2.5])
    assert np.array_equal(O.gelu_fwd(x, "relu"), [0.0, 0.0, 0.0, 1e-9, 2.5])
    assert np.array_equal(O.gelu_grad(x, "relu"), [0.0, 0.0, 0.0, 1.0, 1.0])
    xs = np.linspace(-4, 4, 81) + 0.013                      # away from the kink
    assert np.array_equal(O.gelu_fwd(xs, "relu") - O.gelu_fwd(-xs, "relu"), xs)      # relu(x) - relu(-x) = x
    assert np.array_equal(O.gelu_fwd(xs, "relu"), xs * O.gelu_grad(xs, "relu"))      # relu(x) = x relu'(x)


def test_gelu_erf_against_math_erf_and_torch():
    xs = [-3.0, -1.0, -0.25, 0.5, 1.0, 2.0]
    for v in xs:
        ref = 0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0)))
        assert abs(O.gelu_fwd(np.array([v]), "erf")[0] - ref) < 1e-15
    # textbook value: gelu(1) = Phi(1) = 0.841344746...
    assert abs(O.gelu_fwd(np.array([1.0]), "erf")[0] - 0.8413447460685429) < 1e-15
    torch = pytest.importorskip("torch")
    x = np.linspace(-4, 4, 33)
    for kind, approx in (("erf", "none"), ("tanh", "tanh")):
        t = torch.nn.functional.gelu(torch.tensor(x), approximate=approx).numpy()
        assert np.allclose(O.gelu_fwd(x, kind), t, atol=1e-12)


# ---------------------------------------------------------------- attention
def _brute_attention(qkv, B, S, nh, causal):
    """Scalar-loop softmax attention for tiny inputs."""
    T, H3 = qkv.shape
    H = H3 // 3
    dh = H // nh
    out = np.zeros((T, H)); lse = np.zeros((B, nh, S))
    for b in range(B):
        for h in range(nh):
            for i in range(S):
                q = qkv[b * S + i, h * dh:(h + 1) * dh]
                js = range(i + 1) if causal else range(S)
                sc = [sum(q[d] * qkv[b * S + j, H + h * dh + d] for d in range(dh)) / math.sqrt(dh) for j in js]
                z = sum(math.exp(s) for s in sc)
                lse[b, h, i] = math.log(z)
                for d in range(dh):
                    out[b * S + i, h * dh + d] = sum(
                        math.exp(s) / z * qkv[b * S + j, 2 * H + h * dh + d] for s, j in zip(sc, js))
    return out, lse


@pytest.mark.parametrize("causal", [False, True])
def test_attention_fwd_brute_force(causal):
    B, S, nh, dh = 2, 5, 2, 4
    qkv = rng.normal(size=(B * S, 3 * nh * dh))
    o, lse = O.attention_fwd(qkv, B, S, nh, causal)
    o2, lse2 = _brute_attention(qkv, B, S, nh, causal)
    assert np.allclose(o, o2, atol=1e-12) and np.allclose(lse, lse2, atol=1e-12)


def test_attention_special_cases():
    B, S, nh, dh = 1, 6, 2, 4
    H = nh * dh
    qkv = rng.normal(size=(B * S, 3 * H))
    # causal row 0 attends only to itself: O_0 = V_0 exactly
    o, _ = O.attention_fwd(qkv, B, S, nh, True)
    assert np.array_equal(o[0], qkv[0, 2 * H:])
    # Q = 0 -> uniform weights: mean of V (prefix mean when causal)
    z = qkv.copy(); z[:, :H] = 0
    o, lse = O.attention_fwd(z, B, S, nh, False)
    assert np.allclose(o, np.broadcast_to(z[:, 2 * H:].mean(axis=0), o.shape))
    assert np.allclose(lse, math.log(S))
    o, lse = O.attention_fwd(z, B, S, nh, True)
    pref = np.cumsum(z[:, 2 * H:], axis=0) / np.arange(1, S + 1)[:, None]
    assert np.allclose(o, pref)
    assert np.allclose(lse[0, 0], np.log(np.arange(1, S + 1)))
    # large logits must not overflow
    big = qkv.copy(); big[:, :2 * H] *= 40.0
    o, lse = O.attention_fwd(big, B, S, nh, False)
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(lse))
    # adding a constant vector to every key shifts each row's logits by a
    # per-row constant: output unchanged
    sh = qkv.copy(); sh[:, H:2 * H] += rng.normal(size=H)
    o1, _ = O.attention_fwd(qkv, B, S, nh, False)
    o2, _ = O.attention_fwd(sh, B, S, nh, False)
    assert np.allclose(o1, o2, atol=1e-12)


@pytest.mark.parametrize("causal", [False, True])
def test_attention_matches_torch_autograd(causal):
    torch = pytest.importorskip("torch")
    B, S, nh, dh = 2, 7, 3, 4
    H = nh * dh
    qkv = rng.normal(size=(B * S, 3 * H)); do = rng.normal(size=(B * S, H))
    t = torch.tensor(qkv, requires_grad=True)
    q, k, v = (t[:, i * H:(i + 1) * H].reshape(B, S, nh, dh).permute(0, 2, 1, 3) for i in range(3))
    to = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=causal)
    to = to.permute(0, 2, 1, 3).reshape(B * S, H)
    to.backward(torch.tensor(do))
    o, _ = O.attention_fwd(qkv, B, S, nh, causal)
    d = O.attention_bwd(do, qkv, B, S, nh, causal)
    assert np.allclose(o, to.detach().numpy(), atol=1e-12)
    assert np.allclose(d, t.grad.numpy(), atol=1e-12)


def test_attention_bwd_row_sums_vanish():
    # sum_j dA_ij = 0: the gradient w.r.t. a constant added to all keys' logits of one row
    # is zero -> dK summed against a vector that shifts all logits equally... checked through
    # dQ: adding c*q-independent shift leaves O fixed, so d/dc = 0 for k += c*u (any u):
    B, S, nh, dh = 1, 5, 1, 4
    H = nh * dh
    qkv = rng.normal(size=(S, 3 * H)); do = rng.normal(size=(S, H))
    d = O.attention_bwd(do, qkv, B, S, nh, False)
    dk = d[:, H:2 * H]
    # shifting every key by the same u changes nothing => sum_j dK_j = 0
    assert np.allclose(dk.sum(axis=0), 0, atol=1e-12)


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_closed_forms_and_its_layernorm_special_case():
    rows, cols = 5, 16
    x = rng.normal(size=(rows, cols)) * 3 + 1.0
    g = 1 + 0.1 * rng.normal(size=cols); b = 0.1 * rng.normal(size=cols)
    y, mu, r = O.rmsnorm_fwd(x, g, b, 1e-6)
    assert np.array_equal(mu, np.zeros(rows))
    xh = (y - b) / g
    assert np.allclose((xh * xh).mean(axis=1), 1.0, atol=1e-5)                 # unit mean square per row
    assert np.allclose(xh * np.sqrt((x * x).mean(axis=1) + 1e-6)[:, None], x)   # a pure rescaling of x
    # scaling a row leaves y unchanged (eps -> 0); a constant row a gives sign(a)
    y2, _, _ = O.rmsnorm_fwd(x * 7.5, g, b, 1e-12)
    assert np.allclose(y2, O.rmsnorm_fwd(x, g, b, 1e-12)[0], atol=1e-9)
    yc, _, _ = O.rmsnorm_fwd(np.full((1, cols), -2.0), np.ones(cols), np.zeros(cols), 0.0)
    assert np.allclose(yc, -1.0)
    # on rows whose mean is zero RMSNorm and LayerNorm are the same function, forward and backward
    z = x - x.mean(axis=1, keepdims=True)
    ya, ma, ra = O.layernorm_fwd(z, g, b, 1e-5)
    yb, mb, rb = O.rmsnorm_fwd(z, g, b, 1e-5)
    assert np.allclose(ya, yb, atol=1e-13) and np.allclose(ra, rb, atol=1e-13)
    dy = rng.normal(size=(rows, cols))
    dxa, dga, dba = O.layernorm_bwd(dy, z, ma, ra, g)
    dxb, dgb, dbb = O.rmsnorm_bwd(dy, z, mb, rb, g)
    assert np.allclose(dga, dgb, atol=1e-12) and np.array_equal(dba, dbb)
    # ... except that LayerNorm's dx also projects out the row mean, which RMSNorm's does not
    assert np.allclose(dxa, dxb - (dxb.mean(axis=1, keepdims=True)), atol=1e-12)


def test_rmsnorm_bwd_central_differences_and_torch():
    rows, cols = 4, 12
    x = rng.normal(size=(rows, cols)) + 0.7
    g = 1 + 0.1 * rng.normal(size=cols); b = 0.1 * rng.normal(size=cols); dy = rng.normal(size=(rows, cols))
    y, mu, r = O.rmsnorm_fwd(x, g, b, 1e-5)
    dx, dg, db = O.rmsnorm_bwd(dy, x, mu, r, g)
    f = lambda x_, g_, b_: float((O.rmsnorm_fwd(x_, g_, b_, 1e-5)[0] * dy).sum())
    h = 1e-6
    for arr, grad, which in ((x, dx, 0), (g, dg, 1), (b, db, 2)):
        num = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            a, c = arr.copy(), arr.copy()
            a[idx] += h; c[idx] -= h
            args = [x, g, b]
            args[which] = a; fa = f(*args)
            args[which] = c; fc = f(*args)
            num[idx] = (fa - fc) / (2 * h)
        assert np.allclose(num, grad, atol=1e-8), which
    # orthogonality: dx is orthogonal to x in every row (the output does not change along x, for eps -> 0)
    y0, m0, r0 = O.rmsnorm_fwd(x, g, b, 0.0)
    assert np.allclose((O.rmsnorm_bwd(dy, x, m0, r0, g)[0] * x).sum(axis=1), 0, atol=1e-12)
    torch = pytest.importorskip("torch")
    if hasattr(torch.nn.functional, "rms_norm"):
        tx = torch.tensor(x, requires_grad=True); tg = torch.tensor(g, requires_grad=True)
        ty = torch.nn.functional.rms_norm(tx, (cols,), tg, 1e-5) + torch.tensor(b)
        ty.backward(torch.tensor(dy))
        assert np.allclose(y, ty.detach().numpy(), atol=1e-12)
        assert np.allclose(dx, tx.grad.numpy(), atol=1e-12) and np.allclose(dg, tg.grad.numpy(), atol=1e-12)
