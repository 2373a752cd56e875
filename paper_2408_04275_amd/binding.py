"""ctypes binding of libmmtrain.so: same names as include/mmtrain.h, argument marshalling only.

PyTorch appears here only as the owner of device memory (`tensor.data_ptr()`) and
of the current HIP stream.  Every step of the layer runs in the library's kernels.
If the library has not been built, loading fails loudly: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmmtrain.so")

OK, ERR_INVALID_ARG, ERR_BAD_SEGMENTS, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, ERR_TOO_LARGE = 0, -1, -2, -3, -4, -5, -6
NOALLOC_MAX_TOKENS, NOALLOC_MAX_HEAD_TOKENS = 16384, 64 * 16384
F32, BF16 = 0, 1
DECODER, ENCODER = 0, 1
MASK_CAUSAL, MASK_BIDIR = 0, 1
GEMM_NT, GEMM_NN, GEMM_TN = 0, 1, 2
BWD_ACCUMULATE_WGRAD = 1
BWD_WGRAD_F32 = 2
STACK_RECOMPUTE = 256
GEMM_ACCUMULATE = 1

EXPORTS = ("mmtrain_layer_ctx_bytes", "mmtrain_layer_workspace_bytes", "mmtrain_layer_fwd", "mmtrain_layer_bwd",
           "mmtrain_status_string", "mmtrain_gemm", "mmtrain_gemm_workspace_bytes", "mmtrain_attn_workspace_bytes", "mmtrain_attn_fwd",
           "mmtrain_attn_bwd", "mmtrain_profile_enable", "mmtrain_profile_read", "mmtrain_intra_reorder", "mmtrain_adam_step",
           "mmtrain_stack_ctx_bytes", "mmtrain_stack_workspace_bytes", "mmtrain_stack_fwd", "mmtrain_stack_bwd",
           "mmtrain_pipeline_1f1b", "mmtrain_inter_reorder", "mmtrain_profile_attn_busy",
           "mmtrain_profile_gemm_clock", "mmtrain_attn_bwd_noalloc")
PROF_GEMM_NT, PROF_GEMM_NN, PROF_GEMM_TN, PROF_ATTN_FWD, PROF_ATTN_BWD = range(5)
PROF_NORM_FWD, PROF_NORM_BWD, PROF_ROPE, PROF_ACT_FWD, PROF_ACT_BWD = range(5, 10)

WEIGHT_FIELDS = ("norm1_w", "norm1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                 "norm2_w", "norm2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


class LayerDesc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("kind", C.c_int32), ("dtype", C.c_int32), ("hidden", C.c_int32),
                ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("ffn_hidden", C.c_int32), ("norm_eps", C.c_float), ("rope_base", C.c_float),
                ("softmax_scale", C.c_float)]


class AdamDesc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float), ("grad_scale", C.c_float), ("step", C.c_int32),
                ("zero_grad", C.c_int32)]


def make_adam_desc(lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, grad_scale=1.0, step=1, zero_grad=False):
    return AdamDesc(C.sizeof(AdamDesc), lr, beta1, beta2, eps, weight_decay, grad_scale, step, 1 if zero_grad else 0)


class Batch(C.Structure):
    _fields_ = [("total_tokens", C.c_int32), ("n_segments", C.c_int32), ("cu_seqlens_dev", C.c_void_p),
                ("cu_seqlens_host", C.c_void_p), ("mask_mode", C.c_int32), ("seg_mask_dev", C.c_void_p),
                ("seg_mask_host", C.c_void_p)]


class Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


class Grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


_lib = None


def load_library() -> C.CDLL:
    """Load libmmtrain.so and declare its signatures.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2408_04275_amd.build). "
                           "There is no fallback path.")
    lib = C.CDLL(LIB_PATH)
    P, I, U, S = C.c_void_p, C.c_int32, C.c_uint32, C.c_size_t
    lib.mmtrain_layer_ctx_bytes.restype = S
    lib.mmtrain_layer_ctx_bytes.argtypes = [P, I]
    lib.mmtrain_layer_workspace_bytes.restype = S
    lib.mmtrain_layer_workspace_bytes.argtypes = [P, I, I, C.c_int]
    lib.mmtrain_layer_fwd.restype = C.c_int
    lib.mmtrain_layer_fwd.argtypes = [P, P, P, P, P, P, P, S, P]
    lib.mmtrain_layer_bwd.restype = C.c_int
    lib.mmtrain_layer_bwd.argtypes = [P, P, P, P, P, P, P, P, U, P, S, P]
    lib.mmtrain_stack_ctx_bytes.restype = S
    lib.mmtrain_stack_ctx_bytes.argtypes = [P, I, I, U]
    lib.mmtrain_stack_workspace_bytes.restype = S
    lib.mmtrain_stack_workspace_bytes.argtypes = [P, I, I, I, C.c_int, U]
    lib.mmtrain_stack_fwd.restype = C.c_int
    lib.mmtrain_stack_fwd.argtypes = [P, I, P, P, P, P, P, U, P, S, P]
    lib.mmtrain_stack_bwd.restype = C.c_int
    lib.mmtrain_stack_bwd.argtypes = [P, I, P, P, P, P, P, P, P, U, P, S, P]
    lib.mmtrain_status_string.restype = C.c_char_p
    lib.mmtrain_status_string.argtypes = [C.c_int]
    lib.mmtrain_gemm.restype = C.c_int
    lib.mmtrain_gemm.argtypes = [I, I, I, I, I, P, I, P, I, P, I, P, P, U, P, S, P]
    lib.mmtrain_gemm_workspace_bytes.restype = S
    lib.mmtrain_gemm_workspace_bytes.argtypes = [I, I, I]
    lib.mmtrain_attn_workspace_bytes.restype = S
    lib.mmtrain_attn_workspace_bytes.argtypes = [I, I, I]
    lib.mmtrain_attn_fwd.restype = C.c_int
    lib.mmtrain_attn_fwd.argtypes = [P, P, P, P, P, P, S, P]
    lib.mmtrain_attn_bwd.restype = C.c_int
    lib.mmtrain_attn_bwd.argtypes = [P, P, P, P, P, P, P, P, S, P]
    lib.mmtrain_attn_bwd_noalloc.restype = C.c_int
    lib.mmtrain_attn_bwd_noalloc.argtypes = [P, P, P, P, P, P, P, P]
    lib.mmtrain_profile_enable.restype = None
    lib.mmtrain_profile_enable.argtypes = [C.c_int]
    lib.mmtrain_profile_attn_busy.restype = None
    lib.mmtrain_profile_attn_busy.argtypes = [P]
    lib.mmtrain_profile_gemm_clock.restype = None
    lib.mmtrain_profile_gemm_clock.argtypes = [P]
    lib.mmtrain_profile_read.restype = C.c_int
    lib.mmtrain_profile_read.argtypes = [I, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.c_int]
    lib.mmtrain_adam_step.restype = C.c_int
    lib.mmtrain_adam_step.argtypes = [P, C.c_int64, P, P, P, P, P, I, P]
    lib.mmtrain_intra_reorder.restype = C.c_int
    lib.mmtrain_intra_reorder.argtypes = [P, I, I, P, P, P]
    lib.mmtrain_pipeline_1f1b.restype = C.c_int
    lib.mmtrain_pipeline_1f1b.argtypes = [P, P, I, I, P, C.POINTER(C.c_double), P]
    lib.mmtrain_inter_reorder.restype = C.c_int
    lib.mmtrain_inter_reorder.argtypes = [P, P, I, I, P, P, P, C.POINTER(C.c_int32)]
    _lib = lib
    return lib


# ----------------------------------------------------------------------------
# marshalling helpers
# ----------------------------------------------------------------------------
def _ptr(t) -> Optional[int]:
    """Device/host address of a torch tensor, numpy array, int or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream


def make_desc(kind, dtype, hidden, n_heads, n_kv_heads, head_dim, ffn_hidden, norm_eps=1e-5, rope_base=10000.0,
              softmax_scale=0.0) -> LayerDesc:
    return LayerDesc(C.sizeof(LayerDesc), kind, dtype, hidden, n_heads, n_kv_heads, head_dim, ffn_hidden,
                     norm_eps, rope_base, softmax_scale)


class PackedBatch:
    """Holds the host and device copies of cu_seqlens / per-segment mask modes and the C struct that points at them."""

    def __init__(self, cu_host: np.ndarray, seg_mask_host: Optional[np.ndarray] = None, mask_mode: int = MASK_CAUSAL,
                 cu_dev=None, seg_mask_dev=None, total_tokens: Optional[int] = None):
        self.cu_host = np.ascontiguousarray(cu_host, dtype=np.int32)
        self.seg_mask_host = None if seg_mask_host is None else np.ascontiguousarray(seg_mask_host, dtype=np.uint8)
        self.cu_dev, self.seg_mask_dev = cu_dev, seg_mask_dev
        n_seg = len(self.cu_host) - 1
        T = int(self.cu_host[-1]) if total_tokens is None else total_tokens
        self.struct = Batch(T, n_seg, _ptr(cu_dev), _ptr(self.cu_host), mask_mode, _ptr(seg_mask_dev),
                            _ptr(self.seg_mask_host))

    @classmethod
    def on_device(cls, cu_host, seg_mask_host=None, mask_mode=MASK_CAUSAL, device="cuda"):
        import torch
        cu_host = np.ascontiguousarray(cu_host, dtype=np.int32)
        cu_dev = torch.from_numpy(cu_host).to(device)
        sm_dev = None
        if seg_mask_host is not None:
            seg_mask_host = np.ascontiguousarray(seg_mask_host, dtype=np.uint8)
            sm_dev = torch.from_numpy(seg_mask_host).to(device) if len(seg_mask_host) else torch.empty(1, dtype=torch.uint8, device=device)
        return cls(cu_host, seg_mask_host, mask_mode, cu_dev, sm_dev)


def make_weights(tensors: Dict[str, object]) -> Weights:
    return Weights(*[_ptr(tensors.get(n)) for n in WEIGHT_FIELDS])


def make_grads(tensors: Dict[str, object]) -> Grads:
    return Grads(*[_ptr(tensors.get(n)) for n in WEIGHT_FIELDS])


# ----------------------------------------------------------------------------
# the C-ABI calls, same names
# ----------------------------------------------------------------------------
def mmtrain_status_string(status: int) -> str:
    return load_library().mmtrain_status_string(status).decode()


def mmtrain_adam_step(desc, n, master, grad, exp_avg, exp_avg_sq, param_out, param_dtype, stream=None) -> int:
    return load_library().mmtrain_adam_step(_ref(desc), n, _ptr(master), _ptr(grad), _ptr(exp_avg), _ptr(exp_avg_sq),
                                            _ptr(param_out), param_dtype, _stream(stream))


def mmtrain_intra_reorder(sizes, m: int):
    """Algorithm 1 through the C ABI.  Returns (status, order[n], group_begin[m+1], group_load[m]) as numpy arrays."""
    import numpy as np
    sizes = np.ascontiguousarray(sizes, dtype=np.float64)
    n = int(sizes.shape[0])
    order = np.full(n, -1, dtype=np.int32)
    begin = np.full(max(m, 0) + 1, -1, dtype=np.int32)
    load = np.zeros(max(m, 0), dtype=np.float64)
    rc = load_library().mmtrain_intra_reorder(sizes.ctypes.data if n else None, n, m, order.ctypes.data if n else None,
                                              begin.ctypes.data, load.ctypes.data if m > 0 else None)
    return rc, order, begin, load


def _stage_times(t):
    import numpy as np
    t = np.ascontiguousarray(t, dtype=np.float64)
    if t.ndim != 2:
        raise ValueError("stage times must be [p, l]")
    return t


def mmtrain_pipeline_1f1b(fwd, bwd, order=None):
    """1F1B timeline through the C ABI.  fwd, bwd: [p, l].  Returns (status, makespan, intervals[l])."""
    import numpy as np
    fwd, bwd = _stage_times(fwd), _stage_times(bwd)
    p, l = fwd.shape
    if order is not None:
        order = np.ascontiguousarray(order, dtype=np.int32)
    makespan = C.c_double(-1.0)
    intervals = np.full(l, -1.0, dtype=np.float64)
    rc = load_library().mmtrain_pipeline_1f1b(fwd.ctypes.data if l else None, bwd.ctypes.data if l else None, p, l,
                                              order.ctypes.data if order is not None and l else None, C.byref(makespan),
                                              intervals.ctypes.data if l else None)
    return rc, makespan.value, intervals


def mmtrain_inter_reorder(fwd, bwd, sizes=None):
    """Algorithm 2 through the C ABI.  fwd, bwd: [p, l]; sizes: [l] or None (first + last stage).
    Returns (status, order[l], intervals_seen)."""
    import numpy as np
    fwd, bwd = _stage_times(fwd), _stage_times(bwd)
    p, l = fwd.shape
    if sizes is not None:
        sizes = np.ascontiguousarray(sizes, dtype=np.float64)
        if sizes.shape != (l,):
            raise ValueError("sizes must be [l]")
    order = np.full(l, -1, dtype=np.int32)
    seen = np.full(l, -1.0, dtype=np.float64)
    n = C.c_int32(0)
    rc = load_library().mmtrain_inter_reorder(fwd.ctypes.data if l else None, bwd.ctypes.data if l else None, p, l,
                                              sizes.ctypes.data if sizes is not None and l else None,
                                              order.ctypes.data if l else None, seen.ctypes.data if l else None, C.byref(n))
    return rc, order, seen[:n.value]


def mmtrain_layer_ctx_bytes(desc: Optional[LayerDesc], total_tokens: int) -> int:
    return load_library().mmtrain_layer_ctx_bytes(C.byref(desc) if desc is not None else None, total_tokens)


def mmtrain_layer_workspace_bytes(desc: Optional[LayerDesc], total_tokens: int, n_segments: int, is_bwd: int) -> int:
    return load_library().mmtrain_layer_workspace_bytes(C.byref(desc) if desc is not None else None, total_tokens,
                                                        n_segments, is_bwd)


def _ref(s):
    return None if s is None else C.byref(s)


def mmtrain_layer_fwd(desc, batch, weights, x, y, ctx, workspace, workspace_bytes, stream=None) -> int:
    b = batch.struct if isinstance(batch, PackedBatch) else batch
    return load_library().mmtrain_layer_fwd(_ref(desc), _ref(b), _ref(weights), _ptr(x), _ptr(y), _ptr(ctx),
                                            _ptr(workspace), workspace_bytes, _stream(stream))


def mmtrain_layer_bwd(desc, batch, weights, x, dy, ctx, dx, grads, flags, workspace, workspace_bytes,
                      stream=None) -> int:
    b = batch.struct if isinstance(batch, PackedBatch) else batch
    return load_library().mmtrain_layer_bwd(_ref(desc), _ref(b), _ref(weights), _ptr(x), _ptr(dy), _ptr(ctx),
                                            _ptr(dx), _ref(grads), flags, _ptr(workspace), workspace_bytes,
                                            _stream(stream))


def _array(structs, ctype):
    """A host array of C structures from a list (None stays None)."""
    if structs is None:
        return None
    return structs if isinstance(structs, C.Array) else (ctype * len(structs))(*structs)


def mmtrain_stack_ctx_bytes(desc, n_layers: int, total_tokens: int, flags: int = 0) -> int:
    return load_library().mmtrain_stack_ctx_bytes(_ref(desc), n_layers, total_tokens, flags)


def mmtrain_stack_workspace_bytes(desc, n_layers: int, total_tokens: int, n_segments: int, is_bwd: int,
                                  flags: int = 0) -> int:
    return load_library().mmtrain_stack_workspace_bytes(_ref(desc), n_layers, total_tokens, n_segments, is_bwd, flags)


def mmtrain_stack_fwd(desc, n_layers, batch, weights, x, y, ctx, flags, workspace, workspace_bytes, stream=None) -> int:
    b = batch.struct if isinstance(batch, PackedBatch) else batch
    return load_library().mmtrain_stack_fwd(_ref(desc), n_layers, _ref(b), _array(weights, Weights), _ptr(x), _ptr(y),
                                            _ptr(ctx), flags, _ptr(workspace), workspace_bytes, _stream(stream))


def mmtrain_stack_bwd(desc, n_layers, batch, weights, x, dy, ctx, dx, grads, flags, workspace, workspace_bytes,
                      stream=None) -> int:
    b = batch.struct if isinstance(batch, PackedBatch) else batch
    return load_library().mmtrain_stack_bwd(_ref(desc), n_layers, _ref(b), _array(weights, Weights), _ptr(x), _ptr(dy),
                                            _ptr(ctx), _ptr(dx), _array(grads, Grads), flags, _ptr(workspace),
                                            workspace_bytes, _stream(stream))


def mmtrain_gemm_workspace_bytes(layout: int, M: int, N: int) -> int:
    return load_library().mmtrain_gemm_workspace_bytes(layout, M, N)


def mmtrain_gemm(dtype, layout, M, N, K, A, lda, B, ldb, Cmat, ldc, bias=None, residual=None, flags=0,
                 workspace=None, workspace_bytes=0, stream=None) -> int:
    return load_library().mmtrain_gemm(dtype, layout, M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(Cmat), ldc,
                                       _ptr(bias), _ptr(residual), flags, _ptr(workspace), workspace_bytes,
                                       _stream(stream))


def mmtrain_attn_workspace_bytes(total_tokens: int, n_segments: int, n_heads: int) -> int:
    return load_library().mmtrain_attn_workspace_bytes(total_tokens, n_segments, n_heads)


def mmtrain_attn_fwd(desc, batch, qkv, o, lse, workspace, workspace_bytes, stream=None) -> int:
    b = batch.struct if isinstance(batch, PackedBatch) else batch
    return load_library().mmtrain_attn_fwd(_ref(desc), _ref(b), _ptr(qkv), _ptr(o), _ptr(lse), _ptr(workspace),
                                           workspace_bytes, _stream(stream))


def mmtrain_attn_bwd(desc, batch, qkv, o, lse, d_o, d_qkv, workspace, workspace_bytes, stream=None) -> int:
    b = batch.struct if isinstance(batch, PackedBatch) else batch
    return load_library().mmtrain_attn_bwd(_ref(desc), _ref(b), _ptr(qkv), _ptr(o), _ptr(lse), _ptr(d_o),
                                           _ptr(d_qkv), _ptr(workspace), workspace_bytes, _stream(stream))


def mmtrain_attn_bwd_noalloc(desc, batch, qkv, o, lse, d_o, d_qkv, stream=None) -> int:
    b = batch.struct if isinstance(batch, PackedBatch) else batch
    return load_library().mmtrain_attn_bwd_noalloc(_ref(desc), _ref(b), _ptr(qkv), _ptr(o), _ptr(lse), _ptr(d_o),
                                                   _ptr(d_qkv), _stream(stream))


PROF_ALL = 0x3ff


def mmtrain_profile_enable(class_mask) -> None:
    """Bit k of class_mask enables the event timing of class PROF_* = k; True = all classes, False / 0 = off."""
    if class_mask is True:
        class_mask = PROF_ALL
    load_library().mmtrain_profile_enable(int(class_mask))


def mmtrain_profile_attn_busy(counters) -> None:
    """counters: a zeroed device tensor of 3 x 1024 int64 (rows: forward, dQ, dK/dV), or None to switch off."""
    load_library().mmtrain_profile_attn_busy(None if counters is None else counters.data_ptr())


def mmtrain_profile_gemm_clock(counters) -> None:
    """counters: a device tensor of 4 int64 (shader-clock and 100 MHz counters at the start and end of the first workgroup of
    the last bf16 GEMM launch), or None to switch off."""
    load_library().mmtrain_profile_gemm_clock(None if counters is None else counters.data_ptr())


def gemm_clock_mhz(counters):
    """Shader clock in MHz from the four counters mmtrain_profile_gemm_clock fills (None if no launch wrote them)."""
    c = [int(v) for v in counters.cpu().tolist()]
    return 100.0 * (c[2] - c[0]) / (c[3] - c[1]) if c[3] > c[1] else None


def mmtrain_profile_read(kind: int, reset: bool = True):
    """(total milliseconds, launches) of one kernel class since the last reset."""
    ms, n = C.c_double(0.0), C.c_int64(0)
    rc = load_library().mmtrain_profile_read(kind, C.byref(ms), C.byref(n), 1 if reset else 0)
    if rc != OK:
        raise RuntimeError(f"mmtrain_profile_read: {mmtrain_status_string(rc)}")
    return ms.value, n.value
