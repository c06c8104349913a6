"""CPU oracle for a decoder stage with cross-attention (the second workload shape: T5 is one
of the models of Section 5.1; the paper gives no layer formulas, the textbook ones are written
out here).

TEST INFRASTRUCTURE ONLY: nothing in the product path imports this file, and it imports
nothing from the product.

A layer is the pre-LN transformer layer of oracle/stage.py with a cross-attention block
between its self-attention and its feed-forward block; `mem` [B*S_mem, H] is the encoder's
output, the same for every layer of the stage:

  r1 = x  + SelfAttn(LN1(x) Wqkv + bqkv) Wo + bo
  rc = r1 + CrossAttn(LNc(r1) Wq + bq, mem Wkv + bkv) Wo_c + bo_c
  y  = rc + GELU(LN2(rc) W1 + b1) W2 + b2

The step returns, besides Y, dX and the parameter gradients, dMem: the sum over the layers of
the gradient that reaches `mem` through each layer's key/value projection.  Recompute and swap
(Section 1; Appendix C.2) leave these numbers untouched, so there is no plan executor here: the
device results under any plan are compared with this one definition.

Pins (tests/test_oracle_decoder.py): central differences in float64 for x, mem and every
parameter; with Wo_c = 0 and bo_c = 0 the stage is the plain pre-LN stage of oracle/stage.py
(outputs and shared gradients equal, dMem = 0); samples do not see each other's memory;
dMem is additive over layers; with dropout, central differences again (the masks are fixed functions of
position) and the masks' own pins in tests/test_oracle_dropout.py and tests/test_oracle_cross_attention.py.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from . import dropout as _dropout
from . import stage as _ops

CROSS_WEIGHTS = ("lnc_g", "lnc_b", "w_qc", "b_qc", "w_kvc", "b_kvc", "w_oc", "b_oc")


class DecoderStage:
    def __init__(self, n_layers, hidden, n_heads, ffn, seq, mem_seq, micro_batch, causal=True, gelu="erf", eps=1e-5,
                 p_attn=0.0, p_hidden=0.0, norm="layer"):
        self.L, self.H, self.nh, self.F = n_layers, hidden, n_heads, ffn
        self.S, self.Sm, self.B = seq, mem_seq, micro_batch
        self.causal, self.gelu, self.eps = bool(causal), gelu, eps
        # dropout as in oracle/stage.py (masks from oracle/dropout.py, a function of seed, micro-batch number,
        # layer, site and position): on both attentions' probabilities and on the outputs of the three
        # projections that end in a residual add
        self.p_attn, self.p_hidden = float(p_attn), float(p_hidden)
        self.rng = (0, 0)
        self.norm_fwd, self.norm_bwd = _ops.NORMS[norm]      # LayerNorm, or T5's RMSNorm

    def set_rng(self, seed: int, mb: int):
        self.rng = (int(seed), int(mb))

    def _keeps(self, l):
        """(keep(b) of the self-attention, keep(b) of the cross-attention, their scale), or (None, None, 1)."""
        if self.p_attn == 0.0:
            return None, None, 1.0
        seed, mb = self.rng
        return (lambda b: _dropout.keep_attention(seed, mb, l, b, self.nh, self.S, self.p_attn),
                lambda b: _dropout.keep_cross_attention(seed, mb, l, b, self.nh, self.S, self.Sm, self.p_attn),
                _dropout.scale(self.p_attn))

    def _drop(self, a, l, site):
        if self.p_hidden == 0.0:
            return a
        seed, mb = self.rng
        keep = _dropout.keep_hidden(seed, mb, l, site, a.shape[0], a.shape[1], self.p_hidden)
        return a * (keep.astype(a.dtype) * a.dtype.type(_dropout.scale(self.p_hidden)))

    def layer_fwd(self, x, mem, w, l=0):
        ks, kc, sc = self._keeps(l)
        s = {"X_IN": x}
        s["LN1_OUT"], *s["LN1_STATS"] = self.norm_fwd(x, w["ln1_g"], w["ln1_b"], self.eps)
        s["QKV"] = _ops.linear_fwd(s["LN1_OUT"], w["w_qkv"], w["b_qkv"])
        s["ATTN_OUT"], _ = _ops.attention_fwd(s["QKV"], self.B, self.S, self.nh, self.causal, ks, sc)
        s["RES1"] = x + self._drop(_ops.linear_fwd(s["ATTN_OUT"], w["w_o"], w["b_o"]), l, _dropout.SITE_PROJ)
        s["LNC_OUT"], *s["LNC_STATS"] = self.norm_fwd(s["RES1"], w["lnc_g"], w["lnc_b"], self.eps)
        s["Q_C"] = _ops.linear_fwd(s["LNC_OUT"], w["w_qc"], w["b_qc"])
        s["KV_C"] = _ops.linear_fwd(mem, w["w_kvc"], w["b_kvc"])
        s["ATTN_C_OUT"], _ = _ops.cross_attention_fwd(s["Q_C"], s["KV_C"], self.B, self.S, self.Sm, self.nh, kc, sc)
        s["RES_C"] = s["RES1"] + self._drop(_ops.linear_fwd(s["ATTN_C_OUT"], w["w_oc"], w["b_oc"]), l,
                                            _dropout.SITE_CROSS_PROJ)
        s["LN2_OUT"], *s["LN2_STATS"] = self.norm_fwd(s["RES_C"], w["ln2_g"], w["ln2_b"], self.eps)
        s["FC1_OUT"] = _ops.linear_fwd(s["LN2_OUT"], w["w_fc1"], w["b_fc1"])
        s["GELU_OUT"] = _ops.gelu_fwd(s["FC1_OUT"], self.gelu)
        y = s["RES_C"] + self._drop(_ops.linear_fwd(s["GELU_OUT"], w["w_fc2"], w["b_fc2"]), l, _dropout.SITE_FC2)
        return y, s

    def layer_bwd(self, dy, mem, w, s, l=0):
        """Returns (dx, dmem of this layer, parameter gradients).  A dropout site passes the gradient of its
        output through its mask; the residual branch beside it is untouched."""
        ks, kc, sc = self._keeps(l)
        g = {}
        d_gelu, g["w_fc2"], g["b_fc2"] = _ops.linear_bwd(self._drop(dy, l, _dropout.SITE_FC2), s["GELU_OUT"], w["w_fc2"])
        d_f = d_gelu * _ops.gelu_grad(s["FC1_OUT"], self.gelu)
        d_n, g["w_fc1"], g["b_fc1"] = _ops.linear_bwd(d_f, s["LN2_OUT"], w["w_fc1"])
        d_ln, g["ln2_g"], g["ln2_b"] = self.norm_bwd(d_n, s["RES_C"], *s["LN2_STATS"], w["ln2_g"])
        d_rc = dy + d_ln
        d_oc, g["w_oc"], g["b_oc"] = _ops.linear_bwd(self._drop(d_rc, l, _dropout.SITE_CROSS_PROJ), s["ATTN_C_OUT"],
                                                     w["w_oc"])
        d_qc, d_kvc = _ops.cross_attention_bwd(d_oc, s["Q_C"], s["KV_C"], self.B, self.S, self.Sm, self.nh, kc, sc)
        d_mem, g["w_kvc"], g["b_kvc"] = _ops.linear_bwd(d_kvc, mem, w["w_kvc"])
        d_c, g["w_qc"], g["b_qc"] = _ops.linear_bwd(d_qc, s["LNC_OUT"], w["w_qc"])
        d_ln, g["lnc_g"], g["lnc_b"] = self.norm_bwd(d_c, s["RES1"], *s["LNC_STATS"], w["lnc_g"])
        d_r1 = d_rc + d_ln
        d_o, g["w_o"], g["b_o"] = _ops.linear_bwd(self._drop(d_r1, l, _dropout.SITE_PROJ), s["ATTN_OUT"], w["w_o"])
        d_qkv = _ops.attention_bwd(d_o, s["QKV"], self.B, self.S, self.nh, self.causal, ks, sc)
        d_a, g["w_qkv"], g["b_qkv"] = _ops.linear_bwd(d_qkv, s["LN1_OUT"], w["w_qkv"])
        d_ln, g["ln1_g"], g["ln1_b"] = self.norm_bwd(d_a, s["X_IN"], *s["LN1_STATS"], w["ln1_g"])
        return d_r1 + d_ln, d_mem, g


def decoder_step(stage: DecoderStage, weights: List[Dict[str, np.ndarray]], x, mem, dy, dtype=np.float64):
    """Plain forward then backward.  Returns (Y, dX, dMem, per-layer gradient dicts)."""
    weights = [{k: np.asarray(v, dtype=dtype) for k, v in w.items()} for w in weights]
    h, mem = np.asarray(x, dtype=dtype), np.asarray(mem, dtype=dtype)
    saved = []
    for l, w in enumerate(weights):
        h, s = stage.layer_fwd(h, mem, w, l)
        saved.append(s)
    y = h
    d = np.asarray(dy, dtype=dtype)
    d_mem = np.zeros_like(mem)
    grads = [None] * stage.L
    for l in reversed(range(stage.L)):
        d, dm, grads[l] = stage.layer_bwd(d, mem, weights[l], saved[l], l)
        d_mem = d_mem + dm
    return y, d, d_mem, grads
