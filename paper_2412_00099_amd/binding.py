"""ctypes binding of include/moe_cache.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmoe_cache.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python paper_2412_00099_amd/build.py` "
        "(hipcc, gfx950). There is no fallback path."
    )
lib = C.CDLL(LIB_PATH)

MOE_MAX_EXPERTS = 64
MOE_MAX_TOPK = 8
MOE_OK, MOE_EINVAL, MOE_ENOMEM, MOE_EHIP, MOE_ESTATE = 0, -1, -2, -3, -4
MOE_W_FP32, MOE_W_BF16, MOE_W_INT8_PC, MOE_W_INT4_G128 = 0, 1, 2, 3
MOE_A_FP32, MOE_A_BF16 = 0, 1
MOE_DELTA_RUNNING_MEAN, MOE_DELTA_FIXED, MOE_DELTA_TOKEN = 0, 1, 2
MOE_ROUTE_CACHE_PRIOR, MOE_ROUTE_MAX_RANK, MOE_ROUTE_CUMSUM = 0, 1, 2
MOE_POLICY_LRU, MOE_POLICY_FARTHEST = 0, 1

WEIGHT_FMT = {"fp32": MOE_W_FP32, "bf16": MOE_W_BF16, "int8": MOE_W_INT8_PC, "int4": MOE_W_INT4_G128}
ACT_FMT = {"fp32": MOE_A_FP32, "bf16": MOE_A_BF16}


class moe_cache_config_t(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32),
        ("hidden", C.c_int32),
        ("n_experts", C.c_int32),
        ("inter", C.c_int32),
        ("shared_inter", C.c_int32),
        ("top_k", C.c_int32),
        ("top_j", C.c_int32),
        ("capacity", C.c_int32),
        ("weight_fmt", C.c_int32),
        ("act_fmt", C.c_int32),
        ("renormalize", C.c_int32),
        ("delta_mode", C.c_int32),
        ("route_mode", C.c_int32),
        ("max_rank", C.c_int32),
        ("lambda_", C.c_float),
        ("delta_fixed", C.c_float),
        ("cumsum_p", C.c_float),
        ("reserved", C.c_int32),
        ("compute_stream", C.c_void_p),
        ("copy_stream", C.c_void_p),
    ]


class moe_cache_buffers_t(C.Structure):
    _fields_ = [
        ("host_expert_blob", C.POINTER(C.c_void_p)),
        ("slot_pool", C.POINTER(C.c_void_p)),
        ("gate_w", C.POINTER(C.c_void_p)),
        ("shared_blob", C.POINTER(C.c_void_p)),
        ("initial_resident", C.POINTER(C.c_int32)),
        ("n_initial", C.c_int32),
    ]


class moe_route_out_t(C.Structure):
    _fields_ = [
        ("sel_expert", C.c_int32 * MOE_MAX_TOPK),
        ("sel_slot", C.c_int32 * MOE_MAX_TOPK),
        ("sel_weight", C.c_float * MOE_MAX_TOPK),
        ("miss", C.c_int32 * MOE_MAX_TOPK),
        ("evicted", C.c_int32 * MOE_MAX_TOPK),
        ("n_miss", C.c_int32),
        ("token", C.c_int32),
        ("delta", C.c_float),
        ("margin", C.c_float),
        ("logits", C.c_float * MOE_MAX_EXPERTS),
        ("opaque", C.c_uint32 * 4),
    ]


class moe_cache_stats_t(C.Structure):
    _fields_ = [
        (n, C.c_int64)
        for n in ("tokens", "selections", "hits", "misses", "cold_misses", "evictions", "bytes_filled",
                  "lifetime_sum")
    ]


class moe_cache_plan_t(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("grid", "wavefronts", "depth", "packed_bf16_dot", "boundary_in_expert_launch")]


class moe_cache_tables_t(C.Structure):
    _fields_ = [
        ("expert_slot", C.c_int32 * MOE_MAX_EXPERTS),
        ("slot_expert", C.c_int32 * MOE_MAX_EXPERTS),
        ("stamp", C.c_int64 * MOE_MAX_EXPERTS),
        ("delta_sum", C.c_float),
        ("count", C.c_int32),
    ]


_vp = C.c_void_p
lib.moe_blob_bytes.restype = C.c_size_t
lib.moe_blob_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
lib.moe_slot_bytes.restype = C.c_size_t
lib.moe_slot_bytes.argtypes = [C.POINTER(moe_cache_config_t)]
lib.moe_pack_expert.restype = C.c_int
lib.moe_pack_expert.argtypes = [C.c_int32, C.c_int32, C.c_int32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.moe_cache_init.restype = C.c_int
lib.moe_cache_init.argtypes = [C.POINTER(moe_cache_config_t), C.POINTER(moe_cache_buffers_t), C.POINTER(_vp)]
lib.moe_cache_destroy.restype = None
lib.moe_cache_destroy.argtypes = [_vp]
lib.moe_route_step.restype = C.c_int
lib.moe_route_step.argtypes = [_vp, C.c_int32, _vp, _vp, C.POINTER(moe_route_out_t)]
lib.moe_stack_route_step.restype = C.c_int
lib.moe_stack_route_step.argtypes = [_vp, C.c_int32, _vp, _vp, C.c_float, C.c_int32, _vp, _vp, C.POINTER(moe_route_out_t)]
lib.moe_expert_forward.restype = C.c_int
lib.moe_expert_forward.argtypes = [_vp, C.c_int32, _vp, _vp]
lib.moe_route_batch.restype = C.c_int
lib.moe_route_batch.argtypes = [_vp, C.c_int32, _vp, _vp, C.c_int32, C.POINTER(moe_route_out_t)]
lib.moe_expert_forward_batch.restype = C.c_int
lib.moe_expert_forward_batch.argtypes = [_vp, C.c_int32, _vp, _vp, C.c_int32]
lib.moe_expert_forward_static.restype = C.c_int
lib.moe_expert_forward_static.argtypes = [C.c_int32] * 6 + [_vp, C.c_int32, _vp, C.POINTER(C.c_int32), C.POINTER(C.c_float),
                                          _vp, _vp, _vp]
lib.moe_cache_last_route.restype = C.c_int
lib.moe_cache_last_route.argtypes = [_vp, C.c_int32, C.POINTER(moe_route_out_t)]
lib.moe_cache_stats.restype = C.c_int
lib.moe_cache_stats.argtypes = [_vp, C.c_int32, C.POINTER(moe_cache_stats_t)]
lib.moe_cache_tables.restype = C.c_int
lib.moe_cache_tables.argtypes = [_vp, C.c_int32, C.POINTER(moe_cache_tables_t)]
lib.moe_cache_snapshot.restype = C.c_int
lib.moe_cache_snapshot.argtypes = [_vp, C.c_int32, _vp, C.POINTER(C.c_size_t)]
lib.moe_cache_restore.restype = C.c_int
lib.moe_cache_restore.argtypes = [_vp, C.c_int32, _vp, C.c_size_t]
lib.moe_trace_misses.restype = C.c_int
lib.moe_trace_misses.argtypes = [_vp, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _vp, C.c_int32,
                                 C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
lib.moe_cache_plan.restype = C.c_int
lib.moe_cache_plan.argtypes = [_vp, C.POINTER(moe_cache_plan_t)]
lib.moe_cache_set_lambda.restype = C.c_int
lib.moe_cache_set_lambda.argtypes = [_vp, C.c_float]
lib.moe_cache_set_baseline.restype = C.c_int
lib.moe_cache_set_baseline.argtypes = [_vp, C.c_int32, C.c_int32, C.c_float]
lib.moe_cache_reset.restype = C.c_int
lib.moe_cache_reset.argtypes = [_vp]
lib.moe_residual_rmsnorm.restype = C.c_int
lib.moe_residual_rmsnorm.argtypes = [_vp, _vp, _vp, C.c_float, C.c_int32, _vp, C.c_int32, C.c_int32, _vp]
lib.moe_cache_profile.restype = C.c_int
lib.moe_cache_profile.argtypes = [_vp, C.c_int32, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
lib.moe_last_error.restype = C.c_char_p
lib.moe_last_error.argtypes = []

EXPORTS = [
    "moe_blob_bytes", "moe_slot_bytes", "moe_pack_expert", "moe_cache_init", "moe_cache_destroy", "moe_route_step", "moe_stack_route_step",
    "moe_expert_forward", "moe_route_batch", "moe_expert_forward_batch", "moe_expert_forward_static", "moe_cache_last_route", "moe_cache_stats", "moe_cache_tables", "moe_cache_snapshot",
    "moe_cache_restore", "moe_trace_misses", "moe_cache_plan", "moe_cache_set_lambda",
    "moe_cache_set_baseline", "moe_cache_reset", "moe_residual_rmsnorm", "moe_cache_profile", "moe_last_error",
]


class MoEError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where} failed with {code}: {moe_last_error()}")


def _check(code: int, where: str) -> None:
    if code != MOE_OK:
        raise MoEError(code, where)


def moe_last_error() -> str:
    return (lib.moe_last_error() or b"").decode()


def moe_blob_bytes(weight_fmt: int, hidden: int, inter: int) -> int:
    return int(lib.moe_blob_bytes(weight_fmt, hidden, inter))


def moe_slot_bytes(cfg: moe_cache_config_t) -> int:
    return int(lib.moe_slot_bytes(C.byref(cfg)))


def moe_pack_expert(weight_fmt, hidden, inter, gate, up, down, gate_s, up_s, down_s, blob_dev, stream) -> None:
    _check(lib.moe_pack_expert(weight_fmt, hidden, inter, gate, up, down, gate_s, up_s, down_s, blob_dev, stream),
           "moe_pack_expert")


def moe_cache_init(cfg: moe_cache_config_t, bufs: moe_cache_buffers_t) -> int:
    out = _vp()
    _check(lib.moe_cache_init(C.byref(cfg), C.byref(bufs), C.byref(out)), "moe_cache_init")
    return out.value


def moe_cache_destroy(ctx) -> None:
    lib.moe_cache_destroy(ctx)


def moe_route_step(ctx, layer: int, x_dev, logits_dev, out: moe_route_out_t | None = None, wait: bool = True):
    """wait=True: returns the decision (blocking until the host has it); wait=False: enqueue only, returns None."""
    if not wait:
        _check(lib.moe_route_step(ctx, layer, x_dev, logits_dev, None), "moe_route_step")
        return None
    out = moe_route_out_t() if out is None else out
    _check(lib.moe_route_step(ctx, layer, x_dev, logits_dev, C.byref(out)), "moe_route_step")
    return out


def moe_stack_route_step(ctx, layer: int, h_dev, a_dev, perturb: float, carry: int, x_dev, y_dev=None,
                         out: moe_route_out_t | None = None, wait: bool = True):
    if not wait:
        _check(lib.moe_stack_route_step(ctx, layer, h_dev, a_dev, perturb, carry, x_dev, y_dev, None),
               "moe_stack_route_step")
        return None
    out = moe_route_out_t() if out is None else out
    _check(lib.moe_stack_route_step(ctx, layer, h_dev, a_dev, perturb, carry, x_dev, y_dev, C.byref(out)),
           "moe_stack_route_step")
    return out


def moe_expert_forward(ctx, layer: int, x_dev, y_dev) -> None:
    _check(lib.moe_expert_forward(ctx, layer, x_dev, y_dev), "moe_expert_forward")


def moe_route_batch(ctx, layer: int, x_dev, logits_dev, n_tokens: int):
    """Returns the n_tokens routing records of the batch."""
    out = (moe_route_out_t * n_tokens)()
    _check(lib.moe_route_batch(ctx, layer, x_dev, logits_dev, n_tokens, out), "moe_route_batch")
    return list(out)


def moe_expert_forward_batch(ctx, layer: int, x_dev, y_dev, n_tokens: int) -> None:
    _check(lib.moe_expert_forward_batch(ctx, layer, x_dev, y_dev, n_tokens), "moe_expert_forward_batch")


def moe_expert_forward_static(weight_fmt, act_fmt, hidden, inter, shared_inter, top_k, slot_pool_dev, n_slots,
                              shared_blob_dev, sel_slot, sel_weight, x_dev, y_dev, stream) -> None:
    slots = (C.c_int32 * top_k)(*[int(s) for s in sel_slot])
    weights = (C.c_float * top_k)(*[float(w) for w in sel_weight])
    _check(lib.moe_expert_forward_static(weight_fmt, act_fmt, hidden, inter, shared_inter, top_k, slot_pool_dev, n_slots,
                                         shared_blob_dev, slots, weights, x_dev, y_dev, stream),
           "moe_expert_forward_static")


def moe_cache_last_route(ctx, layer: int) -> moe_route_out_t:
    out = moe_route_out_t()
    _check(lib.moe_cache_last_route(ctx, layer, C.byref(out)), "moe_cache_last_route")
    return out


def moe_cache_stats(ctx, layer: int = -1) -> moe_cache_stats_t:
    out = moe_cache_stats_t()
    _check(lib.moe_cache_stats(ctx, layer, C.byref(out)), "moe_cache_stats")
    return out


def moe_cache_tables(ctx, layer: int) -> moe_cache_tables_t:
    out = moe_cache_tables_t()
    _check(lib.moe_cache_tables(ctx, layer, C.byref(out)), "moe_cache_tables")
    return out


def moe_cache_snapshot(ctx, layer: int) -> bytes:
    n = C.c_size_t(0)
    _check(lib.moe_cache_snapshot(ctx, layer, None, C.byref(n)), "moe_cache_snapshot")
    buf = C.create_string_buffer(n.value)
    _check(lib.moe_cache_snapshot(ctx, layer, buf, C.byref(n)), "moe_cache_snapshot")
    return buf.raw[: n.value]


def moe_cache_restore(ctx, layer: int, blob: bytes) -> None:
    _check(lib.moe_cache_restore(ctx, layer, blob, len(blob)), "moe_cache_restore")


def moe_trace_misses(trace, n_experts: int, capacity: int, policy: int = MOE_POLICY_LRU, initial=()):
    """trace: int32 array [T, K] (host).  Returns (misses, lifetime_sum, evictions)."""
    import numpy as np

    tr = np.ascontiguousarray(trace, dtype=np.int32)
    if tr.ndim != 2:
        raise ValueError("trace must be [tokens, top_k]")
    init = np.ascontiguousarray(list(initial), dtype=np.int32)
    m, life, ev = C.c_int64(), C.c_int64(), C.c_int64()
    _check(lib.moe_trace_misses(tr.ctypes.data, tr.shape[0], tr.shape[1], n_experts, capacity, policy,
                                init.ctypes.data if init.size else None, init.size,
                                C.byref(m), C.byref(life), C.byref(ev)), "moe_trace_misses")
    return m.value, life.value, ev.value


def moe_cache_plan(ctx) -> moe_cache_plan_t:
    out = moe_cache_plan_t()
    _check(lib.moe_cache_plan(ctx, C.byref(out)), "moe_cache_plan")
    return out


def moe_cache_set_lambda(ctx, lam: float) -> None:
    _check(lib.moe_cache_set_lambda(ctx, lam), "moe_cache_set_lambda")


def moe_cache_set_baseline(ctx, route_mode: int, max_rank: int = 0, cumsum_p: float = 0.0) -> None:
    _check(lib.moe_cache_set_baseline(ctx, route_mode, max_rank, cumsum_p), "moe_cache_set_baseline")


def moe_cache_reset(ctx) -> None:
    _check(lib.moe_cache_reset(ctx), "moe_cache_reset")


def moe_residual_rmsnorm(h_dev, y_dev, a_dev, perturb: float, carry: int, x_dev, hidden: int, act_fmt: int,
                         stream) -> None:
    _check(lib.moe_residual_rmsnorm(h_dev, y_dev, a_dev, perturb, carry, x_dev, hidden, act_fmt, stream),
           "moe_residual_rmsnorm")


def moe_cache_profile(ctx, enable: int, reset: bool = True):
    avg, n = C.c_double(), C.c_int64()
    _check(lib.moe_cache_profile(ctx, int(enable), int(reset), C.byref(avg), C.byref(n)), "moe_cache_profile")
    return avg.value, n.value
