"""Host-side checks of the C-ABI: the library loads, exports what the header declares, and
rejects bad arguments before any HIP call (so all of this runs without a GPU)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2408_04275_amd import binding as mm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # a 256-aligned non-NULL address that is never dereferenced on an error path


def header_symbols():
    text = open(os.path.join(ROOT, "include", "mmtrain.h")).read()
    return re.findall(r"MMTRAIN_API\s+[\w\s\*]+?\b(mmtrain_\w+)\s*\(", text)


def test_library_exports_every_declared_symbol():
    lib = mm.load_library()
    names = header_symbols()
    assert len(names) == 23 and set(names) == set(mm.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings():
    assert mm.mmtrain_status_string(0) == "ok"
    for s in (-1, -2, -3, -4, -5, -6):
        assert mm.mmtrain_status_string(s) not in ("ok", "unknown status")
    assert mm.mmtrain_status_string(-99) == "unknown status"


def good_desc(**kw):
    a = dict(kind=mm.DECODER, dtype=mm.BF16, hidden=256, n_heads=4, n_kv_heads=2, head_dim=64, ffn_hidden=688)
    a.update(kw)
    return mm.make_desc(**a)


def test_struct_layout_matches_header():
    assert C.sizeof(mm.LayerDesc) == 44
    assert C.sizeof(mm.Weights) == 12 * C.sizeof(C.c_void_p) == C.sizeof(mm.Grads)


def test_size_queries():
    d = good_desc()
    assert mm.mmtrain_layer_ctx_bytes(d, 512) > 512 * 256 * 2 * 3
    assert mm.mmtrain_layer_ctx_bytes(d, 0) >= 0
    assert mm.mmtrain_layer_workspace_bytes(d, 512, 4, 1) > mm.mmtrain_layer_workspace_bytes(d, 512, 4, 0) > 0
    assert mm.mmtrain_layer_ctx_bytes(None, 512) == 0
    assert mm.mmtrain_layer_ctx_bytes(d, -1) == 0
    bad = good_desc()
    bad.struct_size = 12
    assert mm.mmtrain_layer_ctx_bytes(bad, 512) == 0
    assert mm.mmtrain_layer_workspace_bytes(good_desc(head_dim=72), 512, 4, 1) == 0


def fwd(desc, batch, weights=None, x=FAKE, y=FAKE + 256, ctx=FAKE, ws=FAKE, ws_bytes=1 << 40):
    if weights is None:
        weights = mm.Weights(*[FAKE] * 12)
    return mm.mmtrain_layer_fwd(desc, batch, weights, x, y, ctx, ws, ws_bytes, stream=0)


def batch(cu, modes=None, T=None, dev=True, mode=mm.MASK_CAUSAL):
    return mm.PackedBatch(np.asarray(cu, dtype=np.int32), None if modes is None else np.asarray(modes, dtype=np.uint8),
                          mode, FAKE if dev else None, None if modes is None else FAKE, total_tokens=T)


@pytest.mark.parametrize("kw,status", [
    (dict(head_dim=72), mm.ERR_UNSUPPORTED),
    (dict(head_dim=80, dtype=mm.F32), mm.ERR_UNSUPPORTED),
    (dict(head_dim=256), mm.ERR_UNSUPPORTED),
    (dict(n_heads=4, n_kv_heads=3), mm.ERR_UNSUPPORTED),
    (dict(hidden=250), mm.ERR_UNSUPPORTED),
    (dict(ffn_hidden=100), mm.ERR_UNSUPPORTED),
    (dict(kind=mm.ENCODER, n_kv_heads=2), mm.ERR_UNSUPPORTED),
    (dict(kind=7), mm.ERR_INVALID_ARG),
    (dict(dtype=5), mm.ERR_INVALID_ARG),
    (dict(hidden=0), mm.ERR_INVALID_ARG),
    (dict(norm_eps=0.0), mm.ERR_INVALID_ARG),
    (dict(rope_base=0.5), mm.ERR_INVALID_ARG),
])
def test_bad_descriptions(kw, status):
    assert fwd(good_desc(**kw), batch([0, 16])) == status


@pytest.mark.parametrize("cu,T", [([1, 16], 16), ([0, 9, 5, 16], 16), ([0, 8, 16], 17), ([0, 8, 15], 16)])
def test_bad_segments(cu, T):
    assert fwd(good_desc(), batch(cu, T=T)) == mm.ERR_BAD_SEGMENTS


def test_bad_arguments():
    d = good_desc()
    ok = batch([0, 16])
    assert fwd(None, ok) == mm.ERR_INVALID_ARG
    assert mm.mmtrain_layer_fwd(d, None, mm.Weights(*[FAKE] * 12), FAKE, FAKE + 256, FAKE, FAKE, 1 << 40, 0) == mm.ERR_INVALID_ARG
    assert fwd(d, batch([0, 16], mode=3)) == mm.ERR_INVALID_ARG
    assert fwd(d, batch([0, 16], dev=False)) == mm.ERR_INVALID_ARG           # device cu_seqlens missing
    assert fwd(d, batch([0, 8, 16], modes=[0, 2])) == mm.ERR_INVALID_ARG      # unknown per-segment mode
    half = batch([0, 16]); half.struct.seg_mask_host = FAKE                   # host modes without device modes
    assert fwd(d, half) == mm.ERR_INVALID_ARG
    w = mm.Weights(*[FAKE] * 12); w.w_o = None
    assert fwd(d, ok, weights=w) == mm.ERR_INVALID_ARG
    dec_only = mm.Weights(*[FAKE if not (n.endswith("_b") or n.startswith("b_")) else None for n in mm.WEIGHT_FIELDS])
    assert fwd(good_desc(kind=mm.ENCODER, n_kv_heads=4), ok, weights=dec_only) == mm.ERR_INVALID_ARG
    assert fwd(d, ok, x=None) == mm.ERR_INVALID_ARG
    assert fwd(d, ok, x=FAKE, y=FAKE) == mm.ERR_INVALID_ARG                    # x and y alias
    assert fwd(d, ok, ctx=FAKE + 8) == mm.ERR_INVALID_ARG                      # misaligned ctx
    assert fwd(d, ok, ws_bytes=16) == mm.ERR_WORKSPACE
    assert fwd(d, ok, ws=None) == mm.ERR_WORKSPACE


def test_bwd_validation():
    d = good_desc()
    w = mm.Weights(*[FAKE] * 12)
    g = mm.Grads(*[FAKE] * 12)
    args = lambda **k: dict(dict(desc=d, batch=batch([0, 16]), weights=w, x=FAKE, dy=FAKE, ctx=FAKE, dx=FAKE, grads=g,
                                 flags=0, workspace=FAKE, workspace_bytes=1 << 40, stream=0), **k)
    assert mm.mmtrain_layer_bwd(**args(flags=8)) == mm.ERR_INVALID_ARG
    assert mm.mmtrain_layer_bwd(**args(dy=None)) == mm.ERR_INVALID_ARG
    assert mm.mmtrain_layer_bwd(**args(workspace_bytes=1024)) == mm.ERR_WORKSPACE
    assert mm.mmtrain_layer_bwd(**args(batch=batch([0, 20], T=16))) == mm.ERR_BAD_SEGMENTS


def test_misaligned_tensors_are_rejected_on_the_host():
    # a view such as tensor[1:] of a bf16 tensor is 2-byte aligned: the kernels move 16 bytes per lane, so the
    # entry points refuse it instead of launching (no GPU involved: validation precedes every HIP call)
    d = good_desc()
    ok = batch([0, 16])
    assert fwd(d, ok, x=FAKE + 2) == mm.ERR_INVALID_ARG
    assert fwd(d, ok, y=FAKE + 256 + 8) == mm.ERR_INVALID_ARG
    for field in ("norm1_w", "w_qkv", "w_o", "norm2_w", "w_fc1", "w_fc2"):
        w = mm.Weights(*[FAKE] * 12)
        setattr(w, field, FAKE + 4)
        assert fwd(d, ok, weights=w) == mm.ERR_INVALID_ARG, field
    w = mm.Weights(*[FAKE] * 12)
    g = mm.Grads(*[FAKE] * 12)
    args = lambda **k: dict(dict(desc=d, batch=ok, weights=w, x=FAKE, dy=FAKE, ctx=FAKE, dx=FAKE, grads=g,
                                 flags=0, workspace=FAKE, workspace_bytes=1 << 40, stream=0), **k)
    assert mm.mmtrain_layer_bwd(**args(dy=FAKE + 2)) == mm.ERR_INVALID_ARG
    assert mm.mmtrain_layer_bwd(**args(dx=FAKE + 6)) == mm.ERR_INVALID_ARG
    bad_g = mm.Grads(*[FAKE] * 12); bad_g.w_fc1 = FAKE + 2
    assert mm.mmtrain_layer_bwd(**args(grads=bad_g)) == mm.ERR_INVALID_ARG
    # attention operators: required tensors and their alignment are checked before the token tables are enqueued
    big = 1 << 40
    assert mm.mmtrain_attn_fwd(d, ok, FAKE + 2, FAKE, FAKE, FAKE, big, stream=0) == mm.ERR_INVALID_ARG
    assert mm.mmtrain_attn_fwd(d, ok, FAKE, None, FAKE, FAKE, big, stream=0) == mm.ERR_INVALID_ARG
    assert mm.mmtrain_attn_bwd(d, ok, FAKE, FAKE, FAKE, FAKE + 2, FAKE, FAKE, big, stream=0) == mm.ERR_INVALID_ARG
    assert mm.mmtrain_attn_bwd(d, ok, FAKE, FAKE, FAKE, FAKE, None, FAKE, big, stream=0) == mm.ERR_INVALID_ARG


def test_empty_pack_forward_is_a_no_op():
    assert fwd(good_desc(), batch([0], dev=False)) == mm.OK
    assert fwd(good_desc(), batch([0, 0, 0], dev=False)) == mm.OK


def test_gemm_validation():
    g = lambda **k: mm.mmtrain_gemm(**dict(dict(dtype=mm.BF16, layout=mm.GEMM_NT, M=64, N=64, K=64, A=FAKE, lda=64, B=FAKE,
                                                 ldb=64, Cmat=FAKE, ldc=64, stream=0), **k))
    assert g(dtype=9) == mm.ERR_INVALID_ARG
    assert g(layout=3) == mm.ERR_INVALID_ARG
    assert g(M=-1) == mm.ERR_INVALID_ARG
    assert g(A=None) == mm.ERR_INVALID_ARG
    assert g(lda=32) == mm.ERR_INVALID_ARG
    assert g(ldc=8) == mm.ERR_INVALID_ARG
    assert g(K=60, lda=60, ldb=60) == mm.ERR_UNSUPPORTED                       # bf16 rows must be 16-byte multiples
    assert g(M=0) == mm.OK
    assert g(workspace=None, workspace_bytes=1024) == mm.ERR_INVALID_ARG       # bytes without a buffer
    assert g(workspace=FAKE + 16, workspace_bytes=1024) == mm.ERR_INVALID_ARG  # not 256-byte aligned


def test_gemm_workspace_size():
    # nothing to cut: forward layout, outputs that fill whole rounds of 256 tiles, or more than half of the last one
    assert mm.mmtrain_gemm_workspace_bytes(mm.GEMM_NT, 512, 512) == 0
    assert mm.mmtrain_gemm_workspace_bytes(mm.GEMM_NN, 8192, 4096) == 0        # 512 tiles
    assert mm.mmtrain_gemm_workspace_bytes(mm.GEMM_TN, 4096, 11008) == 0       # 688 tiles: 176 in the last round
    assert mm.mmtrain_gemm_workspace_bytes(mm.GEMM_TN, 0, 64) == 0
    # few tiles: 256 / tiles products of M x N in fp32; a partly filled last round: 256 blocks of 256 x 256
    assert mm.mmtrain_gemm_workspace_bytes(mm.GEMM_TN, 1024, 1024) == 16 * 1024 * 1024 * 4
    assert mm.mmtrain_gemm_workspace_bytes(mm.GEMM_TN, 22016, 4096) == 256 * 256 * 256 * 4
    assert mm.mmtrain_gemm_workspace_bytes(mm.GEMM_NN, 8192, 11008) == 256 * 256 * 256 * 4


def test_stack_sizes_and_validation():
    d = good_desc()
    T, S, n = 512, 3, 5
    act = T * d.hidden * 2
    lc = mm.mmtrain_layer_ctx_bytes(d, T)
    assert mm.mmtrain_stack_ctx_bytes(d, n, T, 0) == (n - 1) * act + n * lc
    assert mm.mmtrain_stack_ctx_bytes(d, n, T, mm.STACK_RECOMPUTE) == (n - 1) * act + lc
    lw = mm.mmtrain_layer_workspace_bytes(d, T, S, 1)
    assert mm.mmtrain_stack_workspace_bytes(d, n, T, S, 1, 0) == lw + 2 * act
    assert mm.mmtrain_stack_workspace_bytes(d, n, T, S, 1, mm.STACK_RECOMPUTE) == lw + 3 * act
    assert mm.mmtrain_stack_workspace_bytes(d, n, T, S, 0, 0) == mm.mmtrain_layer_workspace_bytes(d, T, S, 0)
    assert mm.mmtrain_stack_ctx_bytes(d, 0, T, 0) == 0 and mm.mmtrain_stack_ctx_bytes(d, n, T, 7) == 0
    b = batch([0, 200, 512])
    W = [mm.Weights(*[FAKE] * 12)] * n
    big = 1 << 40
    f = lambda **k: mm.mmtrain_stack_fwd(**dict(dict(desc=d, n_layers=n, batch=b, weights=W, x=FAKE, y=FAKE + 256, ctx=FAKE,
                                                      flags=0, workspace=FAKE, workspace_bytes=big, stream=0), **k))
    assert f(n_layers=0) == mm.ERR_INVALID_ARG
    assert f(weights=None) == mm.ERR_INVALID_ARG
    assert f(flags=mm.BWD_ACCUMULATE_WGRAD) == mm.ERR_INVALID_ARG           # a backward flag on the forward call
    assert f(y=FAKE) == mm.ERR_INVALID_ARG                                   # x and y alias
    assert f(workspace_bytes=16) == mm.ERR_WORKSPACE
    g = lambda **k: mm.mmtrain_stack_bwd(**dict(dict(desc=d, n_layers=n, batch=b, weights=W, x=FAKE, dy=FAKE, ctx=FAKE,
                                                      dx=FAKE, grads=None, flags=0, workspace=FAKE, workspace_bytes=big,
                                                      stream=0), **k))
    assert g(flags=1024) == mm.ERR_INVALID_ARG
    assert g(dx=None) == mm.ERR_INVALID_ARG
    assert g(workspace_bytes=mm.mmtrain_layer_workspace_bytes(d, 512, 2, 1)) == mm.ERR_WORKSPACE   # no room for the gradient buffers
    assert f(batch=batch([0], dev=False)) == mm.OK                           # an empty pack is a no-op
