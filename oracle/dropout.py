"""CPU oracle for the dropout masks of the stage step.

TEST INFRASTRUCTURE ONLY: nothing in the product path imports this file, and it imports
nothing from the product.

The paper does not mention dropout (Section 5.1 only names BERT and GPT-2, which apply it to
the attention probabilities and to the outputs of the attention projection and of the second
feed-forward linear).  What matters for the method is that a recomputed tensor (Section 1;
Appendix C.2, "Recomputation") comes out with the same bits as the first time, so the mask
must be a pure function of where an element sits, not a stream that advances: a counter-based
generator.  The one used here, which the HIP kernels implement independently:

  mix(x):  x ^= x >> 16;  x *= 0x7feb352d;  x ^= x >> 15;  x *= 0x846ca68b;  x ^= x >> 16
           (32-bit; the published "lowbias32" integer mixer, a bijection)
  base   = mix(mix(mix(mix(mix(seed_lo ^ 0x9e3779b9) ^ seed_hi) ^ mb_lo) ^ mb_hi) ^ (8*layer + site))
  k0     = mix(base ^ (unit * 0x9e3779b1));   k1 = mix(k0 ^ 0x85ebca6b)
  bits(i): the mixer applied to i ^ k0, with k1 xored in between its two multiplications
  keep(i) = bits(i) >= floor(p * 2^32);   kept values are scaled by 1 / (1 - p)

site 0: attention probabilities, unit = batch * heads + head, i = query * S + key;
site 1 / 2: output of the attention projection / of FC2, unit = 0, i = token * H + column;
site 3: cross-attention probabilities, unit = batch * heads + head, i = query * Sk + key;
site 4: output of the cross-attention block's projection (decoder stages), like sites 1 and 2.
seed is the caller's, mb counts micro-batches (the caller sets or the library increments it).

Pins (tests/test_oracle_dropout.py): the mixer is injective on a large range and has the
published avalanche property; keep rates, pair independence across elements, rows, heads,
layers, sites and micro-batches; p = 0 keeps everything; the stage step with masks agrees
with central differences and with a brute-force attention written element by element.
"""
from __future__ import annotations

import numpy as np

M1, M2 = 0x7FEB352D, 0x846CA68B
U32 = np.uint32
SITE_ATTN, SITE_PROJ, SITE_FC2, SITE_CROSS, SITE_CROSS_PROJ = 0, 1, 2, 3, 4


def mix(x):
    x = np.asarray(x, dtype=np.uint32).copy()
    x ^= x >> U32(16)
    x *= U32(M1)
    x ^= x >> U32(15)
    x *= U32(M2)
    x ^= x >> U32(16)
    return x


def site_base(seed: int, mb: int, layer: int, site: int) -> int:
    s = mix(U32((seed & 0xFFFFFFFF) ^ 0x9E3779B9))
    for word in ((seed >> 32) & 0xFFFFFFFF, mb & 0xFFFFFFFF, (mb >> 32) & 0xFFFFFFFF, (8 * layer + site) & 0xFFFFFFFF):
        s = mix(s ^ U32(word))
    return int(s)


def unit_keys(base: int, unit: int):
    k0 = mix(U32(base) ^ U32((unit * 0x9E3779B1) & 0xFFFFFFFF))
    k1 = mix(k0 ^ U32(0x85EBCA6B))
    return int(k0), int(k1)


def bits(idx, k0: int, k1: int):
    x = np.asarray(idx, dtype=np.uint32) ^ U32(k0)
    x ^= x >> U32(16)
    x *= U32(M1)
    x ^= x >> U32(15)
    x ^= U32(k1)
    x *= U32(M2)
    x ^= x >> U32(16)
    return x


def threshold(p: float) -> int:
    """floor(p * 2^32) with p taken as the float32 the configuration stores."""
    p32 = float(np.float32(p))
    assert 0.0 <= p32 < 1.0
    return int(np.floor(p32 * 4294967296.0))


def scale(p: float) -> float:
    return 1.0 / (1.0 - float(np.float32(p)))


def keep_hidden(seed, mb, layer, site, T, H, p):
    """[T, H] boolean keep mask of a hidden-state dropout site."""
    assert T * H < 2 ** 32
    k0, k1 = unit_keys(site_base(seed, mb, layer, site), 0)
    with np.errstate(over="ignore"):
        return bits(np.arange(T * H, dtype=np.uint32), k0, k1).reshape(T, H) >= U32(threshold(p))


def keep_attention(seed, mb, layer, b, nh, S, p):
    """[nh, S, S] boolean keep mask of sample b's attention probabilities."""
    assert S * S < 2 ** 32
    base = site_base(seed, mb, layer, SITE_ATTN)
    out = np.empty((nh, S, S), dtype=bool)
    idx = np.arange(S * S, dtype=np.uint32)
    with np.errstate(over="ignore"):
        for h in range(nh):
            k0, k1 = unit_keys(base, b * nh + h)
            out[h] = (bits(idx, k0, k1) >= U32(threshold(p))).reshape(S, S)
    return out


def keep_cross_attention(seed, mb, layer, b, nh, Sq, Sk, p):
    """[nh, Sq, Sk] boolean keep mask of sample b's cross-attention probabilities."""
    assert Sq * Sk < 2 ** 32
    base = site_base(seed, mb, layer, SITE_CROSS)
    out = np.empty((nh, Sq, Sk), dtype=bool)
    idx = np.arange(Sq * Sk, dtype=np.uint32)
    with np.errstate(over="ignore"):
        for h in range(nh):
            k0, k1 = unit_keys(base, b * nh + h)
            out[h] = (bits(idx, k0, k1) >= U32(threshold(p))).reshape(Sq, Sk)
    return out
