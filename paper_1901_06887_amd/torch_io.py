"""Glue between torch device tensors and the C ABI: allocation of the caller-owned buffers
and pointer passing.  No arithmetic happens here."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np
import torch

from . import binding as B


@dataclass
class Served:
    labels: torch.Tensor      # int32 [R]
    probs: torch.Tensor       # float32 [R, row_stride]
    logits: torch.Tensor      # float32 [R, row_stride]
    n_classes: torch.Tensor   # int32 [R]


def specs_of(layers) -> list:
    """mt_layer_spec list from objects with kind/act/in_features/out_features/in_h/in_w/stride (and, where they
    have them, ksize/pad/src/src2)."""
    return [B.layer_spec(l.kind, l.act, l.in_features, l.out_features, l.in_h, l.in_w, l.stride,
                         getattr(l, "ksize", 3), getattr(l, "pad", 1), getattr(l, "src", 0), getattr(l, "src2", 0)) for l in layers]


def context_for(tenants: Dict[int, object], dtype: str, max_requests: int, device: int = 0,
                max_tenants: Optional[int] = None, arena_slack: float = 1.05, run_slots: int = 1,
                arena_bytes: Optional[int] = None, cache: bool = False) -> B.Context:
    """A context sized for the given tenant models (objects with .layers/.weights/.biases); the
    sizes come from the library's own account of every model (mt_model_footprint_get)."""
    code = B.MT_F32 if dtype == "f32" else B.MT_BF16
    width, classes, arena = 64, 1, 0
    for m in tenants.values():
        f = B.model_footprint(specs_of(m.layers), code)
        width, classes, arena = max(width, f["min_width"]), max(classes, f["n_classes"]), arena + f["arena_bytes"]
    T = max_tenants if max_tenants is not None else (max(tenants) + 1 if tenants else 1)
    return B.Context(T, max_requests, width, classes, arena_bytes if arena_bytes is not None else int(arena * arena_slack) + (1 << 20),
                     code, device, run_slots, cache)


def register_tenants(ctx: B.Context, tenants: Dict[int, object]):
    for t, m in tenants.items():
        ctx.register_model(int(t), specs_of(m.layers), m.weights, m.biases, getattr(m, "bn", None), getattr(m, "bn_eps", 1e-5))


def to_device(x: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.to(device)


def alloc_outputs(n: int, row_stride: int, device="cuda:0") -> Served:
    return Served(torch.empty(n, dtype=torch.int32, device=device),
                  torch.empty((n, row_stride), dtype=torch.float32, device=device),
                  torch.empty((n, row_stride), dtype=torch.float32, device=device),
                  torch.empty(n, dtype=torch.int32, device=device))


def serve(ctx: B.Context, tenant_ids: torch.Tensor, inputs: torch.Tensor, out: Optional[Served] = None,
          stream: Optional[torch.cuda.Stream] = None, static: bool = False) -> Served:
    """mt_submit_batch + mt_run (mt_run_static with `static`) on the given (or current) stream; returns
    without synchronising."""
    n = int(tenant_ids.numel())
    assert tenant_ids.dtype == torch.int32 and tenant_ids.is_cuda and inputs.is_cuda and inputs.is_contiguous()
    if out is None:
        out = alloc_outputs(n, ctx.cfg.max_classes, inputs.device)
    s = stream if stream is not None else torch.cuda.current_stream(inputs.device)
    ctx.submit_batch(tenant_ids.data_ptr(), inputs.data_ptr(), n, inputs.shape[1])
    (ctx.run_static if static else ctx.run)(s.cuda_stream, out.labels.data_ptr(), out.probs.data_ptr(), out.logits.data_ptr(),
            out.n_classes.data_ptr(), out.labels.numel(), out.probs.shape[1])
    return out
