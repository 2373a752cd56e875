"""Plumbing around the binding: device buffers for one layer and calls of fwd / bwd.

Used by the tests, the smoke check and the benchmark.  It allocates torch tensors,
uploads host arrays in the storage dtype and hands raw pointers to the C-ABI; it
computes nothing itself.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from . import binding as mm
from .workloads import BF16, DECODER, LayerShape, weight_shapes


def torch_dtype(dtype: int):
    return torch.bfloat16 if dtype == BF16 else torch.float32


def to_device(a: np.ndarray, dtype: int, device="cuda") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device=device, dtype=torch_dtype(dtype))


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def check(status: int, what: str):
    if status != mm.OK:
        raise RuntimeError(f"{what} failed: {mm.mmtrain_status_string(status)} ({status})")


class LayerRunner:
    """Owns the device memory of one layer call sequence (weights, grads, ctx, workspace, x/y/dy/dx)."""

    def __init__(self, shape: LayerShape, weights: Dict[str, np.ndarray], cu: np.ndarray,
                 modes: Optional[np.ndarray] = None, mask_mode: int = mm.MASK_CAUSAL, device="cuda",
                 grad_names=None, grads_f32: bool = False):
        self.shape, self.device = shape, device
        self.desc = mm.make_desc(shape.kind, shape.dtype, shape.hidden, shape.n_heads, shape.n_kv_heads,
                                 shape.head_dim, shape.ffn_hidden, shape.norm_eps, shape.rope_base)
        self.batch = mm.PackedBatch.on_device(cu, modes, mask_mode, device)
        self.T = int(cu[-1])
        S = len(cu) - 1
        dt = torch_dtype(shape.dtype)
        self.w = {k: to_device(v, shape.dtype, device) for k, v in weights.items()}
        names = list(weight_shapes(shape)) if grad_names is None else list(grad_names)
        # gradient buffers: the storage dtype, or fp32 main-gradient buffers (then pass BWD_WGRAD_F32 to backward)
        self.g = {k: torch.zeros(weight_shapes(shape)[k], dtype=torch.float32 if grads_f32 else dt, device=device)
                  for k in names}
        self.weights = mm.make_weights(self.w)
        self.grads = mm.make_grads(self.g)
        self.ctx_bytes = mm.mmtrain_layer_ctx_bytes(self.desc, self.T)
        self.ws_bytes = max(mm.mmtrain_layer_workspace_bytes(self.desc, self.T, S, 0),
                            mm.mmtrain_layer_workspace_bytes(self.desc, self.T, S, 1))
        if self.ctx_bytes == 0 or self.ws_bytes == 0:
            raise RuntimeError("layer description rejected by the library")
        self.ctx = torch.empty(self.ctx_bytes, dtype=torch.uint8, device=device)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)
        self.x = torch.empty((self.T, shape.hidden), dtype=dt, device=device)
        self.y = torch.empty_like(self.x)
        self.dy = torch.empty_like(self.x)
        self.dx = torch.empty_like(self.x)

    def set_inputs(self, x: np.ndarray, dy: np.ndarray):
        self.x.copy_(to_device(x, self.shape.dtype, self.device))
        self.dy.copy_(to_device(dy, self.shape.dtype, self.device))

    def forward(self, stream=None) -> int:
        return mm.mmtrain_layer_fwd(self.desc, self.batch, self.weights, self.x, self.y, self.ctx, self.ws,
                                    self.ws_bytes, stream)

    def backward(self, flags: int = 0, stream=None) -> int:
        return mm.mmtrain_layer_bwd(self.desc, self.batch, self.weights, self.x, self.dy, self.ctx, self.dx,
                                    self.grads, flags, self.ws, self.ws_bytes, stream)

    def step(self, flags: int = 0):
        check(self.forward(), "mmtrain_layer_fwd")
        check(self.backward(flags), "mmtrain_layer_bwd")

    def results(self):
        torch.cuda.synchronize()
        return to_host(self.y), to_host(self.dx), {k: to_host(v) for k, v in self.g.items()}


class StackRunner:
    """Device memory and calls for a stack of layers of one shape (one weight dictionary per layer)."""

    def __init__(self, shape: LayerShape, weights_per_layer, cu: np.ndarray, modes: Optional[np.ndarray] = None,
                 mask_mode: int = mm.MASK_CAUSAL, recompute: bool = False, device="cuda", with_grads: bool = True):
        self.shape, self.device, self.n = shape, device, len(weights_per_layer)
        self.flags = mm.STACK_RECOMPUTE if recompute else 0
        self.desc = mm.make_desc(shape.kind, shape.dtype, shape.hidden, shape.n_heads, shape.n_kv_heads,
                                 shape.head_dim, shape.ffn_hidden, shape.norm_eps, shape.rope_base)
        self.batch = mm.PackedBatch.on_device(cu, modes, mask_mode, device)
        self.T = int(cu[-1])
        S = len(cu) - 1
        dt = torch_dtype(shape.dtype)
        self.w = [{k: to_device(v, shape.dtype, device) for k, v in W.items()} for W in weights_per_layer]
        self.g = [{k: torch.zeros(s, dtype=dt, device=device) for k, s in weight_shapes(shape).items()}
                  for _ in range(self.n)] if with_grads else None
        self.weights = [mm.make_weights(w) for w in self.w]
        self.grads = [mm.make_grads(g) for g in self.g] if with_grads else None
        self.ctx_bytes = mm.mmtrain_stack_ctx_bytes(self.desc, self.n, self.T, self.flags)
        self.ws_bytes = max(mm.mmtrain_stack_workspace_bytes(self.desc, self.n, self.T, S, 0, self.flags),
                            mm.mmtrain_stack_workspace_bytes(self.desc, self.n, self.T, S, 1, self.flags))
        if self.ctx_bytes == 0 or self.ws_bytes == 0:
            raise RuntimeError("stack description rejected by the library")
        self.ctx = torch.empty(self.ctx_bytes, dtype=torch.uint8, device=device)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)
        self.x = torch.empty((self.T, shape.hidden), dtype=dt, device=device)
        self.y = torch.empty_like(self.x)
        self.dy = torch.empty_like(self.x)
        self.dx = torch.empty_like(self.x)

    def set_inputs(self, x: np.ndarray, dy: np.ndarray):
        self.x.copy_(to_device(x, self.shape.dtype, self.device))
        self.dy.copy_(to_device(dy, self.shape.dtype, self.device))

    def forward(self, stream=None) -> int:
        return mm.mmtrain_stack_fwd(self.desc, self.n, self.batch, self.weights, self.x, self.y, self.ctx, self.flags,
                                    self.ws, self.ws_bytes, stream)

    def backward(self, flags: int = 0, stream=None) -> int:
        return mm.mmtrain_stack_bwd(self.desc, self.n, self.batch, self.weights, self.x, self.dy, self.ctx, self.dx,
                                    self.grads, self.flags | flags, self.ws, self.ws_bytes, stream)

    def step(self, flags: int = 0):
        check(self.forward(), "mmtrain_stack_fwd")
        check(self.backward(flags), "mmtrain_stack_bwd")

    def results(self):
        torch.cuda.synchronize()
        return to_host(self.y), to_host(self.dx), [{k: to_host(v) for k, v in g.items()} for g in self.g]
