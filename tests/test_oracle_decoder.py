"""Pins for the oracle's decoder stage with cross-attention: central differences for every
input and parameter, the plain pre-LN stage as the special case of a silent cross block,
sample independence of the memory, and additivity of dMem over layers."""
import numpy as np
import pytest

from oracle import decoder as Dc
from oracle import stage as O

rng = np.random.default_rng(5)


def make(L=2, H=8, nh=2, F=16, S=3, Sm=4, B=2):
    st = Dc.DecoderStage(L, H, nh, F, S, Sm, B, causal=True)
    ws = []
    for _ in range(L):
        w = {"ln1_g": 1 + 0.1 * rng.normal(size=H), "ln1_b": 0.1 * rng.normal(size=H),
             "w_qkv": 0.4 * rng.normal(size=(H, 3 * H)), "b_qkv": 0.1 * rng.normal(size=3 * H),
             "w_o": 0.4 * rng.normal(size=(H, H)), "b_o": 0.1 * rng.normal(size=H),
             "ln2_g": 1 + 0.1 * rng.normal(size=H), "ln2_b": 0.1 * rng.normal(size=H),
             "w_fc1": 0.4 * rng.normal(size=(H, F)), "b_fc1": 0.1 * rng.normal(size=F),
             "w_fc2": 0.4 * rng.normal(size=(F, H)), "b_fc2": 0.1 * rng.normal(size=H),
             "lnc_g": 1 + 0.1 * rng.normal(size=H), "lnc_b": 0.1 * rng.normal(size=H),
             "w_qc": 0.4 * rng.normal(size=(H, H)), "b_qc": 0.1 * rng.normal(size=H),
             "w_kvc": 0.4 * rng.normal(size=(H, 2 * H)), "b_kvc": 0.1 * rng.normal(size=2 * H),
             "w_oc": 0.4 * rng.normal(size=(H, H)), "b_oc": 0.1 * rng.normal(size=H)}
        ws.append(w)
    x, mem, dy = rng.normal(size=(B * S, H)), rng.normal(size=(B * Sm, H)), rng.normal(size=(B * S, H))
    return st, ws, x, mem, dy


def test_central_differences_everywhere():
    st, ws, x, mem, dy = make()
    y, dx, dmem, grads = Dc.decoder_step(st, ws, x, mem, dy)
    loss = lambda ws_, x_, m_: float((Dc.decoder_step(st, ws_, x_, m_, dy)[0] * dy).sum())
    eps = 1e-6

    def numeric(arr, rebuild):
        num = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            a, b = arr.copy(), arr.copy()
            a[idx] += eps; b[idx] -= eps
            num[idx] = (loss(*rebuild(a)) - loss(*rebuild(b))) / (2 * eps)
        return num
    assert np.allclose(numeric(x, lambda a: (ws, a, mem)), dx, atol=2e-7)
    assert np.allclose(numeric(mem, lambda a: (ws, x, a)), dmem, atol=2e-7)
    for l in range(st.L):
        for k in ws[l]:
            def rebuild(a, l=l, k=k):
                w2 = [dict(w) for w in ws]
                w2[l][k] = a
                return w2, x, mem
            assert np.allclose(numeric(ws[l][k], rebuild), grads[l][k], atol=2e-7), (l, k)


def test_silent_cross_block_is_the_plain_stage():
    st, ws, x, mem, dy = make(L=2, H=8, nh=2, F=16, S=4, Sm=3, B=2)
    for w in ws:
        w["w_oc"] = np.zeros_like(w["w_oc"]); w["b_oc"] = np.zeros_like(w["b_oc"])
    y, dx, dmem, grads = Dc.decoder_step(st, ws, x, mem, dy)
    plain = O.Stage(st.L, st.H, st.nh, st.F, st.S, st.B, "pre", True, "erf", st.eps)
    y2, dx2, g2 = O.stage_step(plain, [{k: v for k, v in w.items() if k not in Dc.CROSS_WEIGHTS} for w in ws], x, dy)
    assert np.allclose(y, y2, atol=1e-13) and np.allclose(dx, dx2, atol=1e-13)
    assert np.allclose(dmem, 0, atol=1e-14)
    for l in range(st.L):
        for k in g2[l]:
            assert np.allclose(grads[l][k], g2[l][k], atol=1e-12), (l, k)
        # the block's output projection still gets a gradient, the rest of the block none
        assert np.abs(grads[l]["w_oc"]).max() > 1e-3 and np.allclose(grads[l]["w_qc"], 0) and np.allclose(grads[l]["w_kvc"], 0)


def test_memory_of_another_sample_is_not_seen():
    st, ws, x, mem, dy = make()
    y, dx, dmem, _ = Dc.decoder_step(st, ws, x, mem, dy)
    mem2 = mem.copy(); mem2[st.Sm:] = rng.normal(size=(st.Sm, st.H))
    y2, dx2, dmem2, _ = Dc.decoder_step(st, ws, x, mem2, dy)
    assert np.array_equal(y[:st.S], y2[:st.S]) and np.array_equal(dmem[:st.Sm], dmem2[:st.Sm])
    assert not np.allclose(y[st.S:], y2[st.S:])


def test_dmem_is_the_sum_over_layers():
    st, ws, x, mem, dy = make(L=3)
    y, dx, dmem, _ = Dc.decoder_step(st, ws, x, mem, dy)
    # the memory as a separate copy per layer: each copy's gradient by central differences
    eps, total = 1e-6, np.zeros_like(mem)

    def fwd(mems):
        h = x
        for w, m in zip(ws, mems):
            h, _ = st.layer_fwd(h, m, w)
        return float((h * dy).sum())
    for l in range(st.L):
        for idx in np.ndindex(mem.shape):
            a = [mem.copy() for _ in range(st.L)]; b = [mem.copy() for _ in range(st.L)]
            a[l][idx] += eps; b[l][idx] -= eps
            total[idx] += (fwd(a) - fwd(b)) / (2 * eps)
    assert np.allclose(total, dmem, atol=5e-7)


def test_central_differences_with_dropout():
    st, ws, x, mem, dy = make(L=2, H=8, nh=2, F=16, S=3, Sm=4, B=2)
    st = Dc.DecoderStage(st.L, st.H, st.nh, st.F, st.S, st.Sm, st.B, causal=True, p_attn=0.3, p_hidden=0.25)
    st.set_rng(0x1234567, 9)
    y, dx, dmem, grads = Dc.decoder_step(st, ws, x, mem, dy)
    plain = Dc.DecoderStage(st.L, st.H, st.nh, st.F, st.S, st.Sm, st.B, causal=True)
    assert not np.allclose(y, Dc.decoder_step(plain, ws, x, mem, dy)[0])          # the masks do act
    st.set_rng(0x1234567, 10)
    assert not np.allclose(y, Dc.decoder_step(st, ws, x, mem, dy)[0])             # and differ between micro-batches
    st.set_rng(0x1234567, 9)
    loss = lambda ws_, x_, m_: float((Dc.decoder_step(st, ws_, x_, m_, dy)[0] * dy).sum())
    eps = 1e-6

    def numeric(arr, rebuild):
        num = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            a, b = arr.copy(), arr.copy()
            a[idx] += eps; b[idx] -= eps
            num[idx] = (loss(*rebuild(a)) - loss(*rebuild(b))) / (2 * eps)
        return num
    assert np.allclose(numeric(x, lambda a: (ws, a, mem)), dx, atol=3e-7)
    assert np.allclose(numeric(mem, lambda a: (ws, x, a)), dmem, atol=3e-7)
    for l in range(st.L):
        for k in ("w_oc", "b_oc", "w_kvc", "w_qc", "lnc_g", "w_o", "b_fc2", "w_qkv"):
            def rebuild(a, l=l, k=k):
                w2 = [dict(w) for w in ws]
                w2[l][k] = a
                return w2, x, mem
            assert np.allclose(numeric(ws[l][k], rebuild), grads[l][k], atol=3e-7), (l, k)
