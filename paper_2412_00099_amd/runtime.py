"""Memory plumbing around the C ABI: PyTorch allocates device/pinned memory and streams, nothing else.

ExpertStore owns the two tiers of the paper's Fig. 1 as re-targeted here: a pinned host tensor holding
every packed expert of every layer (the slow tier) and, per layer, a device pool of `capacity` slots
(the fast tier), plus the always-resident router matrices and shared experts.  MoEDecoder wraps one
library context.  No arithmetic of the method happens in this file.
"""
from __future__ import annotations

import ctypes as C

import torch

from . import binding as B


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class ExpertStore:
    def __init__(self, *, n_layers, hidden, n_experts, inter, shared_inter, capacity, weight_fmt, act_fmt,
                 device="cuda:0"):
        self.L, self.d, self.N, self.I, self.Is, self.cap = n_layers, hidden, n_experts, inter, shared_inter, capacity
        self.wfmt = B.WEIGHT_FMT[weight_fmt] if isinstance(weight_fmt, str) else weight_fmt
        self.afmt = B.ACT_FMT[act_fmt] if isinstance(act_fmt, str) else act_fmt
        self.device = torch.device(device)
        self.blob_bytes = B.moe_blob_bytes(self.wfmt, hidden, inter)
        if self.blob_bytes == 0:
            raise ValueError(f"unsupported shape: weight_fmt={weight_fmt} hidden={hidden} inter={inter}")
        self.shared_bytes = B.moe_blob_bytes(self.wfmt, hidden, shared_inter) if shared_inter else 0
        self.host = torch.empty((n_layers, n_experts, self.blob_bytes), dtype=torch.uint8, pin_memory=True)
        self.pools = torch.zeros((n_layers, capacity * self.blob_bytes), dtype=torch.uint8, device=self.device)
        act_dtype = torch.float32 if self.afmt == B.MOE_A_FP32 else torch.bfloat16
        self.gate = torch.zeros((n_layers, n_experts, hidden), dtype=act_dtype, device=self.device)
        self.shared = (
            torch.zeros((n_layers, self.shared_bytes), dtype=torch.uint8, device=self.device) if shared_inter else None
        )
        self._staging = torch.zeros(self.blob_bytes, dtype=torch.uint8, device=self.device)

    # ---- filling ---------------------------------------------------------------------------
    def _pack(self, weights: dict, inter: int, out: torch.Tensor):
        parts, scales = [], []
        for name in ("gate", "up", "down"):
            w = weights[name]
            if isinstance(w, tuple):
                q, s = w
                parts.append(q.to(self.device).contiguous())
                scales.append(s.to(self.device).contiguous())
            else:
                parts.append(w.to(self.device).contiguous())
                scales.append(None)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        B.moe_pack_expert(self.wfmt, self.d, inter, _ptr(parts[0]), _ptr(parts[1]), _ptr(parts[2]),
                          _ptr(scales[0]), _ptr(scales[1]), _ptr(scales[2]), _ptr(out), C.c_void_p(stream))
        torch.cuda.current_stream(self.device).synchronize()  # parts/scales may be temporaries

    def put_expert(self, layer: int, expert: int, weights: dict):
        """Pack canonical weights {'gate','up','down'} on the device and store the blob in the host tier."""
        self._pack(weights, self.I, self._staging)
        self.host[layer, expert].copy_(self._staging)

    def put_shared(self, layer: int, weights: dict):
        self._pack(weights, self.Is, self.shared[layer])

    def put_gate(self, layer: int, w: torch.Tensor):
        self.gate[layer].copy_(w)

    def fill_from(self, workload, weight_fn, shared_fn, gate_fn, progress=None):
        """Fill every layer from generator callbacks (layer[, expert]) -> canonical weights on any device."""
        for l in range(self.L):
            self.put_gate(l, gate_fn(workload, l, self.device))
            for e in range(self.N):
                self.put_expert(l, e, weight_fn(workload, l, e, self.device))
            if self.Is:
                self.put_shared(l, shared_fn(workload, l, self.device))
            if progress:
                progress(l)


class MoEDecoder:
    """One library context over an ExpertStore."""

    def __init__(self, store: ExpertStore, *, top_k, top_j=0, lam=0.0, renormalize=False, initial=None,
                 delta_fixed=None, delta_per_token=False, route_mode=B.MOE_ROUTE_CACHE_PRIOR, max_rank=0,
                 cumsum_p=0.0):
        self.store = store
        dev = store.device
        self.compute_stream = torch.cuda.Stream(device=dev)
        self.copy_stream = torch.cuda.Stream(device=dev)
        cfg = B.moe_cache_config_t()
        cfg.n_layers, cfg.hidden, cfg.n_experts = store.L, store.d, store.N
        cfg.inter, cfg.shared_inter = store.I, store.Is
        cfg.top_k, cfg.top_j, cfg.capacity = top_k, top_j, store.cap
        cfg.weight_fmt, cfg.act_fmt = store.wfmt, store.afmt
        cfg.renormalize = int(renormalize)
        assert delta_fixed is None or not delta_per_token
        cfg.delta_mode = (B.MOE_DELTA_FIXED if delta_fixed is not None else
                          B.MOE_DELTA_TOKEN if delta_per_token else B.MOE_DELTA_RUNNING_MEAN)
        cfg.delta_fixed = float(delta_fixed or 0.0)
        cfg.route_mode, cfg.max_rank, cfg.cumsum_p = route_mode, max_rank, cumsum_p
        cfg.lambda_ = float(lam)
        cfg.compute_stream = self.compute_stream.cuda_stream
        cfg.copy_stream = self.copy_stream.cuda_stream
        self.cfg = cfg
        L, N = store.L, store.N
        self._host_ptrs = (C.c_void_p * (L * N))(*[store.host[l, e].data_ptr() for l in range(L) for e in range(N)])
        self._pool_ptrs = (C.c_void_p * L)(*[store.pools[l].data_ptr() for l in range(L)])
        self._gate_ptrs = (C.c_void_p * L)(*[store.gate[l].data_ptr() for l in range(L)])
        self._shared_ptrs = (C.c_void_p * L)(*[store.shared[l].data_ptr() for l in range(L)]) if store.Is else None
        bufs = B.moe_cache_buffers_t()
        bufs.host_expert_blob = self._host_ptrs
        bufs.slot_pool = self._pool_ptrs
        bufs.gate_w = self._gate_ptrs
        bufs.shared_blob = self._shared_ptrs
        if initial:
            n_init = len(initial[0])
            flat = [e for per_layer in initial for e in per_layer]
            assert len(flat) == L * n_init
            self._initial = (C.c_int32 * len(flat))(*flat)
            bufs.initial_resident = self._initial
            bufs.n_initial = n_init
        torch.cuda.synchronize(dev)
        self.ctx = B.moe_cache_init(cfg, bufs)
        self.top_k = top_k

    def close(self):
        if getattr(self, "ctx", None):
            B.moe_cache_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        self.close()

    def route_step(self, layer, x=None, logits=None, out=None, wait=True):
        return B.moe_route_step(self.ctx, layer, _ptr(x), _ptr(logits), out, wait)

    def stack_route_step(self, layer, h, a, perturb, x, carry=True, y=None, out=None, wait=True):
        return B.moe_stack_route_step(self.ctx, layer, _ptr(h), _ptr(a), perturb, int(carry), _ptr(x), _ptr(y), out, wait)

    def expert_forward(self, layer, x, y):
        B.moe_expert_forward(self.ctx, layer, _ptr(x), _ptr(y))

    def route_batch(self, layer, x=None, logits=None):
        n = (x if x is not None else logits).shape[0]
        return B.moe_route_batch(self.ctx, layer, _ptr(x), _ptr(logits), n)

    def expert_forward_batch(self, layer, x, y):
        B.moe_expert_forward_batch(self.ctx, layer, _ptr(x), _ptr(y), x.shape[0])

    def last_route(self, layer):
        return B.moe_cache_last_route(self.ctx, layer)

    def stats(self, layer=-1):
        return B.moe_cache_stats(self.ctx, layer)

    def tables(self, layer):
        return B.moe_cache_tables(self.ctx, layer)

    def snapshot(self, layer) -> bytes:
        return B.moe_cache_snapshot(self.ctx, layer)

    def restore(self, layer, blob: bytes):
        B.moe_cache_restore(self.ctx, layer, blob)

    def plan(self):
        return B.moe_cache_plan(self.ctx)

    def set_lambda(self, lam):
        B.moe_cache_set_lambda(self.ctx, lam)

    def set_baseline(self, route_mode, max_rank=0, cumsum_p=0.0):
        B.moe_cache_set_baseline(self.ctx, route_mode, max_rank, cumsum_p)

    def reset(self):
        B.moe_cache_reset(self.ctx)

    def residual_rmsnorm(self, h, y, a, perturb, x, carry=True):
        B.moe_residual_rmsnorm(_ptr(h), _ptr(y), _ptr(a), perturb, int(carry), _ptr(x), self.store.d, self.store.afmt,
                               C.c_void_p(self.compute_stream.cuda_stream))

    def profile(self, enable, reset=True):
        return B.moe_cache_profile(self.ctx, enable, reset)
