"""ctypes binding of libdpstage.so: argument marshalling only.

Every function here has the name of the C entry point it calls (minus the
`dp_` prefix) and does nothing but turn torch tensors / numpy arrays into the
pointers and sizes the C ABI takes.  torch supplies device memory and the
stream; all computation happens in the library's kernels.  There is no
fallback: a missing library is an ImportError-like RuntimeError.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdpstage.so")

WEIGHT_FIELDS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                 "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")
SLOTS_PER_LAYER = 12
SLOTS_PER_LAYER_CROSS = 19
# a decoder stage's cross-attention block: names in the tensor dicts -> fields of dp_cross_weights / dp_cross_grads
CROSS_FIELDS = (("lnc_g", "ln_g"), ("lnc_b", "ln_b"), ("w_qc", "w_q"), ("b_qc", "b_q"), ("w_kvc", "w_kv"),
                ("b_kvc", "b_kv"), ("w_oc", "w_o"), ("b_oc", "b_o"))
OP_CLASSES = ("gemm_fwd", "gemm_dgrad", "gemm_wgrad", "attn_fwd", "attn_bwd",
              "ln_fwd", "ln_bwd", "gelu_fwd", "gelu_bwd", "reduce", "dropout")
STATUS = {0: "DP_OK", -1: "DP_E_INVAL", -2: "DP_E_PLAN", -3: "DP_E_BUDGET", -4: "DP_E_DEVMEM",
          -5: "DP_E_HOSTMEM", -6: "DP_E_HIP", -7: "DP_E_UNSUPPORTED"}


class DpError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"{STATUS.get(code, code)}: {text}")
        self.code = code
        self.status = STATUS.get(code, str(code))


class StageConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_heads", "ffn", "seq", "micro_batch",
                                         "norm_style", "causal", "gelu_kind", "dtype")] + [("ln_eps", C.c_float), ("p_attn", C.c_float),
                                                                                 ("p_hidden", C.c_float), ("mem_seq", C.c_int32),
                                                                                 ("norm_kind", C.c_int32)]


class LayerPtrs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


class CrossPtrs(C.Structure):
    _fields_ = [(f, C.c_void_p) for _, f in CROSS_FIELDS]


class PlanReport(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("peak_bytes", "live_peak_bytes", "fixed_bytes", "arena_peak_bytes",
                                          "weight_bytes", "grad_bytes", "kept_act_bytes", "swap_out_bytes",
                                          "swap_in_bytes", "host_pinned_bytes")] + \
               [("replay_flops", C.c_double), ("step_flops", C.c_double)] + \
               [(n, C.c_int32) for n in ("n_replayed_ops", "n_swapped_slots", "first_bad_layer", "first_bad_slot",
                                         "n_fallback_launches")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class StepStats(C.Structure):
    _fields_ = [("step_ms", C.c_float), ("fwd_ms", C.c_float), ("bwd_ms", C.c_float)] + \
               [(n, C.c_uint64) for n in ("d2h_bytes", "h2d_bytes", "arena_high_water", "peak_bytes")] + \
               [("n_kernel_launches", C.c_int32), ("n_replayed_ops", C.c_int32)] + \
               [(n, C.c_float) for n in ("replay_ms", "d2h_busy_ms", "h2d_busy_ms", "swap_wait_ms")] + \
               [("n_fallback_launches", C.c_int32)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class CostModel(C.Structure):
    _fields_ = [("fwd_ns", C.c_int64 * 8), ("bwd_ns", C.c_int64 * 8),
                ("d2h_bytes_per_us", C.c_uint64), ("h2d_bytes_per_us", C.c_uint64),
                ("d2h_duplex_bytes_per_us", C.c_uint64), ("h2d_duplex_bytes_per_us", C.c_uint64),
                ("fwd_more_ns", C.c_int64 * 5), ("bwd_more_ns", C.c_int64 * 5)]

    def node_times(self, n_nodes: int = 8):
        """(forward, backward) node times in execution order; thirteen nodes for a decoder layer."""
        f, b = list(self.fwd_ns) + list(self.fwd_more_ns), list(self.bwd_ns) + list(self.bwd_more_ns)
        return f[:n_nodes], b[:n_nodes]

    def as_dict(self):
        return {"fwd_ns": list(self.fwd_ns), "bwd_ns": list(self.bwd_ns),
                "fwd_more_ns": list(self.fwd_more_ns), "bwd_more_ns": list(self.bwd_more_ns),
                "d2h_bytes_per_us": self.d2h_bytes_per_us, "h2d_bytes_per_us": self.h2d_bytes_per_us,
                "d2h_duplex_bytes_per_us": self.d2h_duplex_bytes_per_us,
                "h2d_duplex_bytes_per_us": self.h2d_duplex_bytes_per_us}


class PlanCostReport(C.Structure):
    _fields_ = [("step_ns", C.c_int64), ("peak_bytes", C.c_uint64), ("d2h_bytes", C.c_uint64),
                ("h2d_bytes", C.c_uint64), ("n_replayed_ops", C.c_int32)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class MemoptReport(C.Structure):
    _fields_ = [("feasible", C.c_int32), ("base_ns", C.c_int64), ("moo_ns", C.c_int64), ("peak_bytes", C.c_uint64),
                ("n_free_swaps", C.c_int32), ("n_paid_swaps", C.c_int32), ("n_recomputed", C.c_int32),
                ("validated_peak_bytes", C.c_uint64), ("exact_step_ns", C.c_int64), ("refine_rounds", C.c_int32)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


MEMOPT_VALIDATE = 1

_lib = None


def lib() -> C.CDLL:
    """Loads the library (once).  Fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2505_05856_amd.build` "
                           "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp, i32, u64, sz = C.c_void_p, C.c_int32, C.c_uint64, C.c_size_t
    L.dp_last_error.restype = C.c_char_p
    L.dp_plan_len.restype = sz
    L.dp_plan_len.argtypes = [C.POINTER(StageConfig)]
    L.dp_plan_validate.argtypes = [C.POINTER(StageConfig), vp, sz, u64, C.c_uint32, C.POINTER(PlanReport)]
    L.dp_stage_init.argtypes = [C.POINTER(StageConfig), C.POINTER(LayerPtrs), u64, C.POINTER(vp)]
    L.dp_stage_step.argtypes = [vp, vp, vp, vp, sz, u64, vp, vp, C.POINTER(LayerPtrs), vp, C.POINTER(StepStats)]
    L.dp_stage_forward.argtypes = [vp, C.c_uint32, C.c_uint32, vp, vp, sz, u64, vp, vp]
    L.dp_stage_backward.argtypes = [vp, C.c_uint32, vp, vp, C.POINTER(LayerPtrs), C.c_uint32, vp]
    L.dp_stage_set_rng.argtypes = [vp, u64, u64]
    L.dp_stage_set_cross.argtypes = [vp, C.POINTER(CrossPtrs), vp]
    L.dp_stage_bind_memory.argtypes = [vp, vp, vp, C.POINTER(CrossPtrs)]
    L.dp_stage_set_weights.argtypes = [vp, C.POINTER(LayerPtrs), vp]
    L.dp_stage_weight_versions.argtypes = [vp]
    L.dp_stage_weight_versions.restype = i32
    L.dp_stage_read_saved.argtypes = [vp, C.c_uint32, C.c_uint32, C.c_uint32, vp, sz, vp]
    L.dp_stage_set_profiling.argtypes = [vp, i32]
    L.dp_stage_op_times.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(u64)]
    L.dp_stage_op_flops.argtypes = [vp, C.POINTER(C.c_double)]
    L.dp_stage_set_debug.argtypes = [vp, C.c_uint32]
    L.dp_stage_destroy.argtypes = [vp]
    L.dp_stage_destroy.restype = None
    L.dp_op_workspace_bytes.restype = sz
    L.dp_op_workspace_bytes.argtypes = [i32, i32]
    L.dp_op_layernorm_fwd.argtypes = [i32, i32, i32, C.c_float, vp, vp, vp, vp, vp, vp]
    L.dp_op_layernorm_bwd.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.dp_op_rmsnorm_fwd.argtypes = [i32, i32, i32, C.c_float, vp, vp, vp, vp, vp, vp]
    L.dp_op_rmsnorm_bwd.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.dp_op_gelu_fwd.argtypes = [i32, i32, sz, vp, vp, vp]
    L.dp_op_gelu_bwd.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    L.dp_op_gemm.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    L.dp_op_colsum.argtypes = [i32, i32, i32, vp, vp, vp, vp]
    L.dp_op_colsum_static.argtypes = [i32, i32, i32, vp, vp, vp]
    L.dp_op_attention_fwd.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, vp, vp]
    L.dp_op_attention_bwd.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    L.dp_op_dropout.argtypes = [i32, sz, vp, vp, vp, vp, i32, vp]
    L.dp_op_attention_dropout_fwd.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp]
    L.dp_op_attention_dropout_bwd.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    L.dp_op_cross_attention_fwd.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    L.dp_op_cross_attention_bwd.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.dp_partition.argtypes = [C.POINTER(StageConfig), C.POINTER(CostModel), i32, u64, u64, u64, C.POINTER(C.c_int64),
                               C.POINTER(u64), C.c_uint32, C.POINTER(i32), vp, sz, C.POINTER(PartitionStage),
                               C.POINTER(PartitionReport)]
    L.dp_probe_mfma.argtypes = [vp, sz, i32, C.POINTER(C.c_float), C.POINTER(C.c_float), vp]
    L.dp_plan_cost.argtypes = [C.POINTER(StageConfig), C.POINTER(CostModel), vp, sz, u64, C.POINTER(PlanCostReport)]
    L.dp_plan_generate.argtypes = [C.POINTER(StageConfig), C.POINTER(CostModel), u64, C.c_uint32, u64, C.c_uint32, vp,
                                   sz, C.POINTER(MemoptReport)]
    L.dp_stage_measure_cost_model.argtypes = [vp, vp, vp, vp, vp, C.POINTER(LayerPtrs), vp, i32, C.POINTER(CostModel)]
    for name in ("dp_probe_mfma", "dp_partition", "dp_plan_cost", "dp_plan_generate", "dp_stage_measure_cost_model", "dp_plan_validate", "dp_stage_init", "dp_stage_step", "dp_stage_forward", "dp_stage_backward", "dp_stage_set_weights", "dp_stage_set_rng", "dp_stage_set_cross", "dp_stage_bind_memory", "dp_stage_set_profiling",
                 "dp_stage_op_times", "dp_stage_op_flops", "dp_stage_set_debug", "dp_op_layernorm_fwd", "dp_op_layernorm_bwd",
                 "dp_op_gelu_fwd", "dp_op_gelu_bwd", "dp_op_gemm", "dp_op_colsum", "dp_op_colsum_static", "dp_op_attention_fwd",
                 "dp_op_attention_bwd", "dp_op_dropout", "dp_op_attention_dropout_fwd", "dp_op_attention_dropout_bwd",
                 "dp_op_cross_attention_fwd", "dp_op_cross_attention_bwd",
                 "dp_op_rmsnorm_fwd", "dp_op_rmsnorm_bwd"):
        getattr(L, name).restype = i32
    _lib = L
    return L


def _check(code: int):
    if code != 0:
        raise DpError(code, lib().dp_last_error().decode())


def make_config(n_layers, hidden, n_heads, ffn, seq, micro_batch, norm_style="post", causal=False,
                gelu="erf", dtype="bf16", ln_eps=1e-5, p_attn=0.0, p_hidden=0.0, mem_seq=0, norm="layer") -> StageConfig:
    return StageConfig(n_layers, hidden, n_heads, ffn, seq, micro_batch,
                       {"post": 0, "pre": 1}[norm_style], int(bool(causal)), {"erf": 0, "tanh": 1, "relu": 2}[gelu],
                       {"f32": 0, "bf16": 1}[dtype], ln_eps, p_attn, p_hidden, mem_seq, {"layer": 0, "rms": 1}[norm])


def _plan_buf(plan):
    a = np.ascontiguousarray(np.asarray(plan, dtype=np.uint8))
    return a, a.ctypes.data_as(C.c_void_p), a.size


def plan_len(cfg: StageConfig) -> int:
    return int(lib().dp_plan_len(C.byref(cfg)))


def plan_validate(cfg: StageConfig, plan, budget_bytes: int = 0, inflight: int = 1, raise_on_error=True):
    """Returns (status_code, report dict)."""
    rep = PlanReport()
    if plan is None:
        code = lib().dp_plan_validate(C.byref(cfg), None, 0, budget_bytes, inflight, C.byref(rep))
    else:
        keep, p, n = _plan_buf(plan)
        code = lib().dp_plan_validate(C.byref(cfg), p, n, budget_bytes, inflight, C.byref(rep))
    if raise_on_error:
        _check(code)
    return code, rep.as_dict()


def make_cost_model(fwd_ns, bwd_ns, d2h_bytes_per_us, h2d_bytes_per_us, d2h_duplex=0, h2d_duplex=0) -> CostModel:
    cm = CostModel()
    assert len(fwd_ns) == len(bwd_ns) and len(fwd_ns) in (8, 13)
    for i in range(8):
        cm.fwd_ns[i], cm.bwd_ns[i] = int(fwd_ns[i]), int(bwd_ns[i])
    for i in range(8, len(fwd_ns)):      # a decoder layer's nodes 8..12
        cm.fwd_more_ns[i - 8], cm.bwd_more_ns[i - 8] = int(fwd_ns[i]), int(bwd_ns[i])
    cm.d2h_bytes_per_us, cm.h2d_bytes_per_us = int(d2h_bytes_per_us), int(h2d_bytes_per_us)
    cm.d2h_duplex_bytes_per_us, cm.h2d_duplex_bytes_per_us = int(d2h_duplex), int(h2d_duplex)
    return cm


def plan_cost(cfg: StageConfig, cm: CostModel, plan, fixed_bytes: int = 0):
    keep, p, n = _plan_buf(plan)
    rep = PlanCostReport()
    _check(lib().dp_plan_cost(C.byref(cfg), C.byref(cm), p, n, fixed_bytes, C.byref(rep)))
    return rep.as_dict()


def plan_generate(cfg: StageConfig, cm: CostModel, budget_bytes: int, inflight: int = 1, fixed_bytes: int = 0,
                  flags: int = 0, raise_on_error=True):
    """Returns (status_code, plan as uint8 array, report dict)."""
    n = plan_len(cfg)
    out = np.zeros(n, dtype=np.uint8)
    rep = MemoptReport()
    code = lib().dp_plan_generate(C.byref(cfg), C.byref(cm), budget_bytes, inflight, fixed_bytes, flags,
                                  out.ctypes.data_as(C.c_void_p), n, C.byref(rep))
    if raise_on_error:
        _check(code)
    return code, out, rep.as_dict()


class PartitionStage(C.Structure):
    _fields_ = [("first_layer", C.c_int32), ("n_layers", C.c_int32), ("inflight", C.c_int32), ("used_memopt", C.c_int32),
                ("time_ns", C.c_int64), ("base_ns", C.c_int64), ("moo_ns", C.c_int64), ("peak_bytes", C.c_uint64)]


class PartitionReport(C.Structure):
    _fields_ = [("feasible", C.c_int32), ("any_memopt", C.c_int32), ("time_ns", C.c_int64), ("rho_cb", C.c_int32),
                ("rho_mb", C.c_int32), ("n_memopt", C.c_int32), ("n_positions", C.c_int32)]


def partition(chain_cfg: StageConfig, cm: CostModel, n_stages: int, budget_bytes: int, fixed_per_layer: int,
              fixed_per_stage: int, extra_ns=None, extra_bytes=None, flags: int = 0, raise_on_error=True):
    """dp_partition.  Returns (status, dict): feasible, time_ns, cuts, rho_cb, rho_mb, counters, stages (list of
    dicts with the stage's plan as a uint8 array)."""
    L = chain_cfg.n_layers
    n = plan_len(chain_cfg)
    plan = np.zeros(n, dtype=np.uint8)
    cuts = (C.c_int32 * max(1, n_stages - 1))()
    stages = (PartitionStage * max(1, n_stages))()
    rep = PartitionReport()
    ens = (C.c_int64 * L)(*[int(v) for v in extra_ns]) if extra_ns is not None else None
    eby = (C.c_uint64 * L)(*[int(v) for v in extra_bytes]) if extra_bytes is not None else None
    code = lib().dp_partition(C.byref(chain_cfg), C.byref(cm), n_stages, budget_bytes, fixed_per_layer,
                              fixed_per_stage, ens, eby, flags, cuts, plan.ctypes.data_as(C.c_void_p), n, stages,
                              C.byref(rep))
    if raise_on_error:
        _check(code)
    out = {f: getattr(rep, f) for f, _ in PartitionReport._fields_}
    out["feasible"], out["any_memopt"] = bool(rep.feasible), bool(rep.any_memopt)
    if code in (0, -3):
        out["cuts"] = [int(cuts[i]) for i in range(n_stages - 1)]
        out["stages"] = []
        for x in range(n_stages):
            d = {f: getattr(stages[x], f) for f, _ in PartitionStage._fields_}
            spl = n // L      # plan bytes a layer (more in a decoder stage)
            a = d["first_layer"] * spl
            d["plan"] = plan[a:a + d["n_layers"] * spl].copy()
            d["memopt"] = bool(d.pop("used_memopt"))
            out["stages"].append(d)
    return code, out


def last_error() -> str:
    return lib().dp_last_error().decode()


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _layer_array(layers: Sequence[Dict[str, "object"]]):
    arr = (LayerPtrs * len(layers))()
    for i, d in enumerate(layers):
        for n in WEIGHT_FIELDS:
            setattr(arr[i], n, d[n].data_ptr())
    return arr


def _cross_array(layers: Sequence[Dict[str, "object"]]):
    arr = (CrossPtrs * len(layers))()
    for i, d in enumerate(layers):
        for name, field in CROSS_FIELDS:
            setattr(arr[i], field, d[name].data_ptr())
    return arr


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


class Stage:
    """Owns a dp_stage handle."""

    def __init__(self, handle: int, cfg: StageConfig):
        self.handle, self.cfg = handle, cfg

    def close(self):
        if self.handle:
            lib().dp_stage_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def stage_init(cfg: StageConfig, weights: Sequence[Dict[str, "object"]], arena_bytes_hint: int = 0) -> Stage:
    """weights: per layer, a dict of contiguous device tensors named as WEIGHT_FIELDS."""
    out = C.c_void_p()
    _check(lib().dp_stage_init(C.byref(cfg), _layer_array(weights), arena_bytes_hint, C.byref(out)))
    return Stage(out.value, cfg)


def stage_step(stage: Stage, x_in, dy, plan, budget_bytes, y_out, dx_out, grads: Sequence[Dict[str, "object"]],
               stream=None, want_stats: bool = False):
    keep, p, n = _plan_buf(plan)
    stats = StepStats() if want_stats else None
    _check(lib().dp_stage_step(stage.handle, _ptr(x_in), _ptr(dy), p, n, budget_bytes, _ptr(y_out), _ptr(dx_out),
                               _layer_array(grads), _stream_ptr(stream),
                               C.byref(stats) if want_stats else None))
    return stats.as_dict() if want_stats else None


GRAD_ACCUMULATE = 1


def stage_forward(stage: Stage, slot: int, inflight: int, x_in, plan, budget_bytes, y_out, stream=None):
    keep, p, n = _plan_buf(plan)
    _check(lib().dp_stage_forward(stage.handle, slot, inflight, _ptr(x_in), p, n, budget_bytes, _ptr(y_out),
                                  _stream_ptr(stream)))


def stage_backward(stage: Stage, slot: int, dy, dx_out, grads: Sequence[Dict[str, "object"]], flags: int = 0,
                   stream=None):
    _check(lib().dp_stage_backward(stage.handle, slot, _ptr(dy), _ptr(dx_out), _layer_array(grads), flags,
                                   _stream_ptr(stream)))


def stage_read_saved(stage: Stage, slot: int, layer: int, tensor: int, dst, stream=None):
    """Copies saved tensor `tensor` of layer `layer` of the micro-batch in flight in `slot` into the device
    tensor `dst` (exactly that many bytes)."""
    _check(lib().dp_stage_read_saved(stage.handle, slot, layer, tensor, _ptr(dst), dst.numel() * dst.element_size(),
                                     _stream_ptr(stream)))


def stage_set_weights(stage: Stage, weights: Sequence[Dict[str, "object"]], stream=None):
    _check(lib().dp_stage_set_weights(stage.handle, _layer_array(weights), _stream_ptr(stream)))


def stage_set_cross(stage: Stage, weights: Sequence[Dict[str, "object"]], stream=None):
    """Uploads the cross-attention block's parameters (tensors named as the first column of CROSS_FIELDS)."""
    _check(lib().dp_stage_set_cross(stage.handle, _cross_array(weights), _stream_ptr(stream)))


def stage_bind_memory(stage: Stage, mem, d_mem=None, grads: Optional[Sequence[Dict[str, "object"]]] = None):
    _check(lib().dp_stage_bind_memory(stage.handle, _ptr(mem), _ptr(d_mem) if d_mem is not None else None,
                                      _cross_array(grads) if grads is not None else None))


def stage_set_rng(stage: Stage, seed: int, counter: int):
    _check(lib().dp_stage_set_rng(stage.handle, seed, counter))


def stage_weight_versions(stage: Stage) -> int:
    return int(lib().dp_stage_weight_versions(stage.handle))


def stage_set_profiling(stage: Stage, enabled: bool):
    _check(lib().dp_stage_set_profiling(stage.handle, int(enabled)))


def stage_op_times(stage: Stage):
    ms = (C.c_float * len(OP_CLASSES))()
    cnt = (C.c_uint64 * len(OP_CLASSES))()
    _check(lib().dp_stage_op_times(stage.handle, ms, cnt))
    return {n: (float(ms[i]), int(cnt[i])) for i, n in enumerate(OP_CLASSES)}


def stage_op_flops(stage: Stage):
    f = (C.c_double * len(OP_CLASSES))()
    _check(lib().dp_stage_op_flops(stage.handle, f))
    return {n: f[i] for i, n in enumerate(OP_CLASSES)}


def stage_measure_cost_model(stage: Stage, x_in, dy, y_out, dx_out, grads, steps: int = 3, stream=None) -> CostModel:
    cm = CostModel()
    _check(lib().dp_stage_measure_cost_model(stage.handle, _ptr(x_in), _ptr(dy), _ptr(y_out), _ptr(dx_out),
                                             _layer_array(grads), _stream_ptr(stream), steps, C.byref(cm)))
    return cm


def stage_set_debug(stage: Stage, flags: int):
    _check(lib().dp_stage_set_debug(stage.handle, flags))


# ---------------------------------------------------------------- standalone ops
def _dt(t) -> int:
    import torch
    return {torch.float32: 0, torch.bfloat16: 1}[t.dtype]


def op_workspace_bytes(rows: int, cols: int) -> int:
    return int(lib().dp_op_workspace_bytes(rows, cols))


def op_layernorm_fwd(x, gamma, beta, eps, y, stats, stream=None):
    _check(lib().dp_op_layernorm_fwd(_dt(x), x.shape[0], x.shape[1], eps, _ptr(x), _ptr(gamma), _ptr(beta),
                                     _ptr(y), _ptr(stats), _stream_ptr(stream)))


def op_layernorm_bwd(dy, x, stats, gamma, dres, dx, dgamma, dbeta, ws, dx_colsum=None, stream=None):
    _check(lib().dp_op_layernorm_bwd(_dt(x), x.shape[0], x.shape[1], _ptr(dy), _ptr(x), _ptr(stats), _ptr(gamma),
                                     _ptr(dres), _ptr(dx), _ptr(dgamma), _ptr(dbeta), _ptr(dx_colsum), _ptr(ws),
                                     _stream_ptr(stream)))


def op_rmsnorm_fwd(x, gamma, beta, eps, y, stats, stream=None):
    _check(lib().dp_op_rmsnorm_fwd(_dt(x), x.shape[0], x.shape[1], eps, _ptr(x), _ptr(gamma), _ptr(beta),
                                   _ptr(y), _ptr(stats), _stream_ptr(stream)))


def op_rmsnorm_bwd(dy, x, stats, gamma, dres, dx, dgamma, dbeta, ws, dx_colsum=None, stream=None):
    _check(lib().dp_op_rmsnorm_bwd(_dt(x), x.shape[0], x.shape[1], _ptr(dy), _ptr(x), _ptr(stats), _ptr(gamma),
                                   _ptr(dres), _ptr(dx), _ptr(dgamma), _ptr(dbeta), _ptr(dx_colsum), _ptr(ws),
                                   _stream_ptr(stream)))


def op_gelu_fwd(x, y, kind=0, stream=None):
    _check(lib().dp_op_gelu_fwd(_dt(x), kind, x.numel(), _ptr(x), _ptr(y), _stream_ptr(stream)))


def op_gelu_bwd(dy, x, dx, dbias, ws, kind=0, stream=None):
    _check(lib().dp_op_gelu_bwd(_dt(x), kind, x.shape[0], x.shape[1], _ptr(dy), _ptr(x), _ptr(dx), _ptr(dbias),
                                _ptr(ws), _stream_ptr(stream)))


def op_gemm(mode, M, N, K, A, B, bias, res, Cout, stream=None):
    _check(lib().dp_op_gemm(_dt(A), mode, M, N, K, _ptr(A), _ptr(B), _ptr(bias), _ptr(res), _ptr(Cout),
                            _stream_ptr(stream)))


def op_colsum(x, out, ws, stream=None):
    _check(lib().dp_op_colsum(_dt(x), x.shape[0], x.shape[1], _ptr(x), _ptr(out), _ptr(ws), _stream_ptr(stream)))


def op_colsum_static(x, out, stream=None):
    _check(lib().dp_op_colsum_static(_dt(x), x.shape[0], x.shape[1], _ptr(x), _ptr(out), _stream_ptr(stream)))


def op_attention_fwd(qkv, B, S, nh, dh, causal, o, lse, stream=None):
    _check(lib().dp_op_attention_fwd(_dt(qkv), B, S, nh, dh, int(causal), _ptr(qkv), _ptr(o), _ptr(lse),
                                     _stream_ptr(stream)))


def op_attention_bwd(qkv, o, lse, d_o, B, S, nh, dh, causal, dqkv, ws, stream=None):
    _check(lib().dp_op_attention_bwd(_dt(qkv), B, S, nh, dh, int(causal), _ptr(qkv), _ptr(o), _ptr(lse), _ptr(d_o),
                                     _ptr(dqkv), _ptr(ws), _stream_ptr(stream)))


class Dropout(C.Structure):
    """Which mask: rate, seed, micro-batch number, layer (dp_dropout)."""
    _fields_ = [("p", C.c_float), ("seed", C.c_uint64), ("micro_batch", C.c_uint64), ("layer", C.c_int32)]


SITE_PROJ, SITE_FC2, SITE_CROSS_PROJ = 1, 2, 4


def op_dropout(x, res, y, drop: Dropout, site: int, stream=None):
    _check(lib().dp_op_dropout(_dt(x), x.numel(), _ptr(x), _ptr(res) if res is not None else None, _ptr(y),
                               C.byref(drop), site, _stream_ptr(stream)))


def op_attention_dropout_fwd(qkv, B, S, nh, dh, causal, o, lse, drop: Dropout, stream=None):
    _check(lib().dp_op_attention_dropout_fwd(_dt(qkv), B, S, nh, dh, int(causal), _ptr(qkv),
                                             _ptr(o) if o is not None else None,
                                             _ptr(lse) if lse is not None else None, C.byref(drop),
                                             _stream_ptr(stream)))


def op_attention_dropout_bwd(qkv, o, lse, d_o, B, S, nh, dh, causal, dqkv, ws, drop: Dropout, stream=None):
    _check(lib().dp_op_attention_dropout_bwd(_dt(qkv), B, S, nh, dh, int(causal), _ptr(qkv), _ptr(o), _ptr(lse),
                                             _ptr(d_o), _ptr(dqkv), _ptr(ws), C.byref(drop), _stream_ptr(stream)))


def op_cross_attention_fwd(q, kv, B, Sq, Sk, nh, dh, o, lse, drop: Dropout = None, stream=None):
    _check(lib().dp_op_cross_attention_fwd(_dt(q), B, Sq, Sk, nh, dh, _ptr(q), _ptr(kv),
                                           _ptr(o) if o is not None else None,
                                           _ptr(lse) if lse is not None else None,
                                           C.byref(drop) if drop is not None else None, _stream_ptr(stream)))


def op_cross_attention_bwd(q, kv, o, lse, d_o, B, Sq, Sk, nh, dh, dq, dkv, ws, drop: Dropout = None, stream=None):
    _check(lib().dp_op_cross_attention_bwd(_dt(q), B, Sq, Sk, nh, dh, _ptr(q), _ptr(kv), _ptr(o), _ptr(lse), _ptr(d_o),
                                           _ptr(dq), _ptr(dkv), _ptr(ws),
                                           C.byref(drop) if drop is not None else None, _stream_ptr(stream)))


def probe_mfma(data, iters: int = 20000, stream=None):
    """Matrix-core issue rate (TFLOP/s) and shader clock (MHz) with operand bits from the bf16 tensor `data`."""
    tf, mhz = C.c_float(), C.c_float()
    n = data.numel() // 8 * 8
    _check(lib().dp_probe_mfma(_ptr(data), n, iters, C.byref(tf), C.byref(mhz), _stream_ptr(stream)))
    return float(tf.value), float(mhz.value)
