"""Device-buffer plumbing around the binding for tests and the benchmark:
uploads seeded inputs with torch, allocates outputs, downloads results.
No arithmetic of the method happens here."""
from __future__ import annotations

from typing import Dict, List

import numpy as np
import torch

from . import binding as B


def to_binding_config(cfg) -> B.StageConfig:
    """`cfg` is a synthetic.StageConfig (duck-typed)."""
    return B.make_config(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, cfg.micro_batch,
                         cfg.norm_style, cfg.causal, cfg.gelu, cfg.dtype, cfg.ln_eps, cfg.p_attn, cfg.p_hidden,
                         getattr(cfg, "mem_seq", 0), getattr(cfg, "norm", "layer"))


def torch_dtype(cfg):
    return torch.bfloat16 if cfg.dtype == "bf16" else torch.float32


def upload(a: np.ndarray, cfg, device="cuda:0") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device).to(torch_dtype(cfg)).contiguous()


def download(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


class StageRunner:
    """Holds a stage handle plus its device inputs/outputs."""

    def __init__(self, cfg, weights: List[Dict[str, np.ndarray]], x: np.ndarray, dy: np.ndarray,
                 device="cuda:0", arena_bytes_hint: int = 0, mem: np.ndarray = None):
        self.cfg, self.device = cfg, device
        self.bcfg = to_binding_config(cfg)
        self.w = [{k: upload(v, cfg, device) for k, v in layer.items()} for layer in weights]
        self.x, self.dy = upload(x, cfg, device), upload(dy, cfg, device)
        self.y = torch.empty_like(self.x)
        self.dx = torch.empty_like(self.x)
        self.g = [{k: torch.empty_like(v) for k, v in layer.items()} for layer in self.w]
        self.mem = self.d_mem = None
        torch.cuda.synchronize()
        self.stage = B.stage_init(self.bcfg, self.w, arena_bytes_hint)
        if getattr(cfg, "mem_seq", 0) > 0:   # decoder stage: the block's parameters and the encoder memory
            self.mem = upload(mem, cfg, device)
            self.d_mem = torch.empty_like(self.mem)
            B.stage_set_cross(self.stage, self.w)
            B.stage_bind_memory(self.stage, self.mem, self.d_mem, self.g)

    def poison_outputs(self):
        for t in [self.y, self.dx] + [v for layer in self.g for v in layer.values()] + \
                ([self.d_mem] if self.d_mem is not None else []):
            t.fill_(float("nan"))

    def step(self, plan, budget_bytes: int = 0, want_stats: bool = False, stream=None):
        return B.stage_step(self.stage, self.x, self.dy, plan, budget_bytes, self.y, self.dx, self.g,
                            stream=stream, want_stats=want_stats)

    def results(self):
        torch.cuda.synchronize()
        return download(self.y), download(self.dx), [{k: download(v) for k, v in layer.items()} for layer in self.g]

    def raw_results(self):
        """Bit patterns of every output, for bit-exactness checks."""
        torch.cuda.synchronize()
        outs = [self.y, self.dx] + [layer[k] for layer in self.g for k in B.WEIGHT_FIELDS]
        if self.d_mem is not None:
            outs += [self.d_mem] + [layer[k] for layer in self.g for k, _ in B.CROSS_FIELDS]
        return [t.detach().clone().view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu() for t in outs]

    def close(self):
        self.stage.close()


class ScheduleRunner:
    """A stage handle plus device buffers for several micro-batches, driven event by event
    through dp_stage_forward / dp_stage_backward.  Slot bookkeeping only."""

    def __init__(self, cfg, weights: List[Dict[str, np.ndarray]], xs, dys, device="cuda:0"):
        self.cfg, self.device = cfg, device
        self.bcfg = to_binding_config(cfg)
        self.w = [{k: upload(v, cfg, device) for k, v in layer.items()} for layer in weights]
        self.x = [upload(x, cfg, device) for x in xs]
        self.dy = [upload(d, cfg, device) for d in dys]
        self.y = [torch.empty_like(x) for x in self.x]
        self.dx = [torch.empty_like(x) for x in self.x]
        self.g = [{k: torch.empty_like(v) for k, v in layer.items()} for layer in self.w]
        torch.cuda.synchronize()
        self.stage = B.stage_init(self.bcfg, self.w, 0)
        self.slot_of: Dict[int, int] = {}

    def poison_outputs(self):
        for t in self.y + self.dx + [v for layer in self.g for v in layer.values()]:
            t.fill_(float("nan"))

    def forward(self, m: int, inflight: int, plan, budget_bytes: int = 0, stream=None):
        slot = min(s for s in range(inflight + 1) if s not in self.slot_of.values())
        B.stage_forward(self.stage, slot, inflight, self.x[m], plan, budget_bytes, self.y[m], stream=stream)
        self.slot_of[m] = slot

    def backward(self, m: int, accumulate: bool, stream=None):
        slot = self.slot_of.pop(m)
        B.stage_backward(self.stage, slot, self.dy[m], self.dx[m], self.g, B.GRAD_ACCUMULATE if accumulate else 0,
                         stream=stream)

    def run(self, order, inflight: int, plan, budget_bytes: int = 0):
        """`order`: ("F", m) / ("B", m) events; `plan` one plan or one per micro-batch.
        The first backward overwrites the gradients, the later ones accumulate."""
        first = True
        for kind, m in order:
            if kind == "F":
                self.forward(m, inflight, plan[m] if isinstance(plan, (list, tuple)) else plan, budget_bytes)
            else:
                self.backward(m, accumulate=not first)
                first = False

    def results(self):
        torch.cuda.synchronize()
        return ([download(t) for t in self.y], [download(t) for t in self.dx],
                [{k: download(v) for k, v in layer.items()} for layer in self.g])

    def raw_results(self):
        torch.cuda.synchronize()
        outs = self.y + self.dx + [layer[k] for layer in self.g for k in B.WEIGHT_FIELDS]
        return [t.detach().clone().view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu() for t in outs]

    def close(self):
        self.stage.close()


def steady_state_ms(run: "StageRunner", plan, inflight: int, budget_bytes: int, warmup: int, steps: int) -> float:
    """Milliseconds per micro-batch in the steady state of a one-forward-one-backward schedule with
    `inflight` micro-batches between forward and backward: the backward of the oldest, then the forward of
    the next into the slot it left, gradients accumulating.  Timing and slot bookkeeping only."""
    import time
    k, st = inflight, run.stage
    for s in range(k):
        B.stage_forward(st, s, k, run.x, plan, budget_bytes, run.y)

    def turn(i):
        B.stage_backward(st, i % k, run.dy, run.dx, run.g, B.GRAD_ACCUMULATE if i else 0)
        B.stage_forward(st, i % k, k, run.x, plan, budget_bytes, run.y)
    for i in range(warmup):
        turn(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        turn(warmup + i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    for s in range(k):
        B.stage_backward(st, s, run.dy, run.dx, run.g, B.GRAD_ACCUMULATE)
    torch.cuda.synchronize()
    return ms
