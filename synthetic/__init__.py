"""Seeded synthetic inputs for a pipeline-stage training step.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds no arithmetic of the method itself: only the stage
configurations, a counter-based random generator, bf16 rounding of inputs and
the plan byte arrays (which are *data* handed to either side).

The paper (Section 5.1) names its workloads only as BERT (340 M), GPT-2 (770 M)
and so on, with no dataset, sequence length or precision; the configurations
below are the stand-ins this build measures on.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List

import numpy as np

# ----------------------------------------------------------------------------
# plan vocabulary: one action byte per saved tensor ("slot") of every layer.
# The paper's plan granularity is the tensor (Section 4.3: candidates are the
# entries of each node's saved-tensor list).
# ----------------------------------------------------------------------------
KEEP, RECOMPUTE, SWAP = 0, 1, 2

SLOT_NAMES = (
    "X_IN", "LN1_STATS", "LN1_OUT", "QKV", "ATTN_LSE", "ATTN_OUT",
    "RES1", "LN2_STATS", "LN2_OUT", "FC1_OUT", "GELU_OUT", "RES2",
)
SLOTS_PER_LAYER = len(SLOT_NAMES)
# a decoder stage (mem_seq > 0) has seven more saved tensors a layer, after those above
CROSS_SLOT_NAMES = ("LNC_STATS", "LNC_OUT", "Q_C", "KV_C", "ATTN_C_LSE", "ATTN_C_OUT", "RES_C")
SLOT = {n: i for i, n in enumerate(SLOT_NAMES + CROSS_SLOT_NAMES)}

WEIGHT_NAMES = (
    "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2",
)
CROSS_WEIGHT_NAMES = ("lnc_g", "lnc_b", "w_qc", "b_qc", "w_kvc", "b_kvc", "w_oc", "b_oc")


@dataclass(frozen=True)
class StageConfig:
    n_layers: int
    hidden: int
    n_heads: int
    ffn: int
    seq: int
    micro_batch: int
    norm_style: str = "post"   # "post" (BERT-style) or "pre" (GPT-2-style)
    causal: bool = False
    gelu: str = "erf"          # feed-forward activation: GELU as "erf" or "tanh", or "relu"
    dtype: str = "bf16"        # "f32" or "bf16"
    ln_eps: float = 1e-5
    p_attn: float = 0.0        # dropout rate on the attention probabilities
    p_hidden: float = 0.0      # dropout rate after the attention projection and after FC2
    mem_seq: int = 0           # > 0: decoder stage, cross-attention over an encoder memory of this length
    norm: str = "layer"        # what the normalisations compute: "layer" (LayerNorm) or "rms" (RMSNorm)

    @property
    def slots_per_layer(self) -> int:
        return SLOTS_PER_LAYER + (len(CROSS_SLOT_NAMES) if self.mem_seq > 0 else 0)

    @property
    def mem_tokens(self) -> int:
        return self.micro_batch * self.mem_seq

    @property
    def tokens(self) -> int:
        return self.micro_batch * self.seq

    @property
    def head_dim(self) -> int:
        return self.hidden // self.n_heads

    def alias_slots(self) -> tuple:
        """Slots that are another layer's X_IN (or the stage output) and own no
        storage in this norm style; their plan bytes are ignored."""
        return (SLOT["RES2"],) if self.norm_style == "pre" else (SLOT["LN2_OUT"],)

    def weight_shapes(self) -> Dict[str, tuple]:
        H, F = self.hidden, self.ffn
        return {
            "ln1_g": (H,), "ln1_b": (H,), "w_qkv": (H, 3 * H), "b_qkv": (3 * H,),
            "w_o": (H, H), "b_o": (H,), "ln2_g": (H,), "ln2_b": (H,),
            "w_fc1": (H, F), "b_fc1": (F,), "w_fc2": (F, H), "b_fc2": (H,),
            "lnc_g": (H,), "lnc_b": (H,), "w_qc": (H, H), "b_qc": (H,),
            "w_kvc": (H, 2 * H), "b_kvc": (2 * H,), "w_oc": (H, H), "b_oc": (H,),
        }

    def model_flops(self) -> float:
        """Algorithmic fwd+bwd FLOP of one step (backward = 2x forward; only the
        lower triangle of a causal attention counts; replay not counted)."""
        T, H, F, S = self.tokens, self.hidden, self.ffn, self.seq
        attn = (2 if self.causal else 4) * T * S * H
        cross = 0
        if self.mem_seq > 0:   # query and output projections, key/value projection of the memory, the attention
            cross = 4 * T * H * H + 4 * self.mem_tokens * H * H + 4 * T * self.mem_seq * H
        return 3.0 * self.n_layers * (8 * T * H * H + 4 * T * H * F + attn + cross)


CONFIGS: Dict[str, StageConfig] = {
    # tiny BERT-style stage, fp32 debug mode
    "C1": StageConfig(1, 128, 2, 512, 64, 2, "post", False, "erf", "f32"),
    # BERT-Large stage (24 layers over 4 stages = 6 layers a stage)
    "C2": StageConfig(6, 1024, 16, 4096, 512, 8, "post", False, "erf", "bf16"),
    # GPT-2-XL-width decoder stage
    "C3": StageConfig(8, 1600, 25, 6400, 1024, 4, "pre", True, "erf", "bf16"),
    # the same stage at micro-batch 32 (40 GB budget)
    "C4": StageConfig(8, 1600, 25, 6400, 1024, 32, "pre", True, "erf", "bf16"),
    # wide decoder stage (64 GB budget)
    "C5": StageConfig(4, 4096, 32, 11008, 2048, 8, "pre", True, "erf", "bf16"),
    # decoder stage of a T5-Large-sized encoder-decoder model (24 decoder layers over 4 stages),
    # cross-attention over an encoder memory as long as the decoder sequence
    "T5": StageConfig(6, 1024, 16, 4096, 512, 8, "pre", True, "erf", "bf16", mem_seq=512),
}
BUDGETS = {"C4": 40 * 10**9, "C5": 64 * 10**9}

# ----------------------------------------------------------------------------
# counter-based generator: splitmix64 of (seed, counter) -> Box-Muller normal
# ----------------------------------------------------------------------------
_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def splitmix64(seed: int, counters: np.ndarray) -> np.ndarray:
    """Output number `counters[i]` (0-based) of the splitmix64 stream of `seed`."""
    with np.errstate(over="ignore"):
        z = np.uint64(seed) + (counters.astype(np.uint64) + np.uint64(1)) * _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def normal(seed: int, offset: int, n: int) -> np.ndarray:
    """n standard normals (float64) from stream `seed`, element i using stream
    positions 2*(offset+i) and 2*(offset+i)+1."""
    out = np.empty(n, dtype=np.float64)
    step = 1 << 22
    for s in range(0, n, step):
        e = min(n, s + step)
        idx = np.arange(offset + s, offset + e, dtype=np.uint64)
        a = splitmix64(seed, idx * np.uint64(2))
        b = splitmix64(seed, idx * np.uint64(2) + np.uint64(1))
        u1 = ((a >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)
        u2 = (b >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
        out[s:e] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return out


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float values to the nearest bf16 (ties to even); returns float32
    holding exactly representable bf16 values."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    bits = bits + np.uint64(0x7FFF) + ((bits >> np.uint64(16)) & np.uint64(1))
    bits = (bits & np.uint64(0xFFFF0000)).astype(np.uint32)
    return bits.view(np.float32).reshape(f.shape)


def _store(cfg: StageConfig, a: np.ndarray) -> np.ndarray:
    a32 = a.astype(np.float32)
    return round_to_bf16(a32) if cfg.dtype == "bf16" else a32


def make_weights(cfg: StageConfig, seed: int = 0, sigma: float = 0.02) -> List[Dict[str, np.ndarray]]:
    """Per-layer weights ~ N(0, sigma), LayerNorm gain = 1 + N(0, sigma); values
    are float32 arrays already rounded to the stage's storage type."""
    layers, off = [], 0
    shapes = cfg.weight_shapes()
    for _ in range(cfg.n_layers):
        w = {}
        for name in WEIGHT_NAMES + (CROSS_WEIGHT_NAMES if cfg.mem_seq > 0 else ()):
            shp = shapes[name]
            n = int(np.prod(shp))
            v = sigma * normal(seed, off, n).reshape(shp)
            off += n
            if name in ("ln1_g", "ln2_g", "lnc_g"):
                v = 1.0 + v
            w[name] = _store(cfg, v)
        layers.append(w)
    return layers


def make_activations(cfg: StageConfig, seed_x: int = 1, seed_dy: int = 2):
    """Stage input X and upstream gradient dY, both [T, H] ~ N(0, 1)."""
    n = cfg.tokens * cfg.hidden
    x = normal(seed_x, 0, n).reshape(cfg.tokens, cfg.hidden)
    dy = normal(seed_dy, 0, n).reshape(cfg.tokens, cfg.hidden)
    return _store(cfg, x), _store(cfg, dy)


def make_memory(cfg: StageConfig, seed: int = 3) -> np.ndarray:
    """Encoder memory of a decoder stage, [micro_batch * mem_seq, H] ~ N(0, 1)."""
    n = cfg.mem_tokens * cfg.hidden
    return _store(cfg, normal(seed, 0, n).reshape(cfg.mem_tokens, cfg.hidden))


def sharpen_attention(cfg: StageConfig, weights, logit_std: float = 4.0):
    """Scale the Q and K column blocks of w_qkv so attention logits have a
    standard deviation near `logit_std` (sigma = 0.02 alone gives an almost
    uniform softmax, which would leave the softmax numerics unexercised)."""
    H = cfg.hidden
    out = []
    for w in weights:
        w = dict(w)
        m = w["w_qkv"].astype(np.float64).copy()
        # q_d, k_d ~ N(0, H*s^2) for unit-variance inputs; logit = sum_d q_d k_d / sqrt(dh)
        s2 = float(np.var(m[:, :H]))
        cur = H * s2  # std of the logit before scaling
        g = np.sqrt(logit_std / max(cur, 1e-30))
        m[:, : 2 * H] *= g
        w["w_qkv"] = _store(cfg, m)
        out.append(w)
    return out


# ----------------------------------------------------------------------------
# plans
# ----------------------------------------------------------------------------
def plan_len(cfg: StageConfig) -> int:
    return cfg.n_layers * cfg.slots_per_layer


def repair_plan(cfg: StageConfig, plan: np.ndarray) -> np.ndarray:
    """Alias slots and the stage input have no producer/storage inside the
    stage: force them to KEEP."""
    p = plan.reshape(cfg.n_layers, cfg.slots_per_layer).copy()
    for s in cfg.alias_slots():
        p[:, s] = KEEP
    p[0, SLOT["X_IN"]] = KEEP
    return p.reshape(-1)


def plan_uniform(cfg: StageConfig, action: int, keep_layer_inputs: bool = False) -> np.ndarray:
    p = np.full((cfg.n_layers, cfg.slots_per_layer), action, dtype=np.uint8)
    if keep_layer_inputs:
        p[:, SLOT["X_IN"]] = KEEP
    return repair_plan(cfg, p.reshape(-1))


def plan_keep_all(cfg):
    return plan_uniform(cfg, KEEP)


def plan_all_recompute(cfg):
    """Every saved tensor regenerated in backward; each layer's input stays
    resident as the checkpoint boundary."""
    return plan_uniform(cfg, RECOMPUTE, keep_layer_inputs=True)


def plan_all_swap(cfg):
    return plan_uniform(cfg, SWAP)


def plan_from_slots(cfg, actions: Dict[str, int]) -> np.ndarray:
    p = np.zeros((cfg.n_layers, cfg.slots_per_layer), dtype=np.uint8)
    for name, a in actions.items():
        p[:, SLOT[name]] = a
    return repair_plan(cfg, p.reshape(-1))


def plan_recompute_attention(cfg):
    return plan_from_slots(cfg, {"QKV": RECOMPUTE, "ATTN_LSE": RECOMPUTE, "ATTN_OUT": RECOMPUTE})


def plan_swap_ffn_recompute_norm_gelu(cfg):
    return plan_from_slots(cfg, {
        "FC1_OUT": SWAP, "LN1_OUT": RECOMPUTE, "LN1_STATS": RECOMPUTE,
        "LN2_OUT": RECOMPUTE, "LN2_STATS": RECOMPUTE, "GELU_OUT": RECOMPUTE})


def plan_seeded(cfg, seed: int) -> np.ndarray:
    """Per-slot action = splitmix64(seed) draw mod 3, in (layer, slot) order."""
    n = plan_len(cfg)
    z = splitmix64(seed, np.arange(n, dtype=np.uint64))
    return repair_plan(cfg, (z % np.uint64(3)).astype(np.uint8))


PLANS = {
    "C1": [("keep-all", plan_keep_all), ("all-recompute", plan_all_recompute)],
    "C2": [("keep-all", plan_keep_all)],
    "C3": [("recompute-attention", plan_recompute_attention)],
    "C4": [("swap-fc1-recompute-ln-gelu", plan_swap_ffn_recompute_norm_gelu)],
    "C5": [("seed7-mixed", lambda c: plan_seeded(c, 7))],
    "T5": [("keep-all", plan_keep_all)],
}


def small_like(cfg: StageConfig, **kw) -> StageConfig:
    """A reduced copy of a configuration (same style, smaller extents)."""
    return replace(cfg, **kw)
