"""GPU parity of the operator-level entry points (GEMM family, attention) against fp64 definitions."""
import numpy as np
import pytest
import torch

from oracle import bf16_storage
from oracle import layer_oracle as orc
from paper_2408_04275_amd import parity
from paper_2408_04275_amd import binding as mm
from paper_2408_04275_amd import workloads as wl
from paper_2408_04275_amd.harness import check, to_device, to_host, torch_dtype
from util import assert_parity

pytestmark = pytest.mark.gpu


def gemm_case(dtype, layout, M, N, K, bias=False, residual=False, accumulate=False, seed=0, workspace=False):
    rng = np.random.default_rng(seed)
    shp_a = (K, M) if layout == mm.GEMM_TN else (M, K)
    shp_b = (N, K) if layout == mm.GEMM_NT else (K, N)
    A = wl.round_to(rng.standard_normal(shp_a), dtype)
    B = wl.round_to(rng.standard_normal(shp_b), dtype)
    C0 = wl.round_to(rng.standard_normal((M, N)), dtype)
    bv = wl.round_to(rng.standard_normal(N), dtype) if bias else None
    R = wl.round_to(rng.standard_normal((M, N)), dtype) if residual else None
    a64 = A.astype(np.float64).T if layout == mm.GEMM_TN else A.astype(np.float64)
    b64 = B.astype(np.float64).T if layout == mm.GEMM_NT else B.astype(np.float64)
    ref = a64 @ b64
    if bias: ref = ref + bv[None, :]
    if residual: ref = ref + R
    if accumulate: ref = ref + C0
    dA, dB, dC = to_device(A, dtype), to_device(B, dtype), to_device(C0, dtype)
    dbias = to_device(bv, dtype) if bias else None
    dR = to_device(R, dtype) if residual else None
    wsb = mm.mmtrain_gemm_workspace_bytes(layout, M, N) if workspace else 0
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda") if wsb else None
    check(mm.mmtrain_gemm(dtype, layout, M, N, K, dA, shp_a[1], dB, shp_b[1], dC, N, dbias, dR,
                          mm.GEMM_ACCUMULATE if accumulate else 0, ws, wsb), "mmtrain_gemm")
    torch.cuda.synchronize()
    got = to_host(dC)
    # one bf16 rounding of the fp32-accumulated result: at most 2^-9 relative per element
    bars = {"max_err": 4e-3, "floor_err": 8e-3, "l2_err": 2.5e-3} if dtype == mm.BF16 else \
        {k: 2e-6 * np.sqrt(max(K, 1)) for k in ("max_err", "floor_err", "l2_err")}
    assert_parity(f"gemm{layout} {M}x{N}x{K}", got, ref, dtype, bars)


SHAPES = [(8, 8, 8), (256, 256, 64), (304, 520, 136), (512, 1376, 256), (264, 248, 688), (1000, 264, 72)]


@pytest.mark.parametrize("layout", [mm.GEMM_NT, mm.GEMM_NN, mm.GEMM_TN])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_bf16(layout, M, N, K):
    gemm_case(mm.BF16, layout, M, N, K)


@pytest.mark.parametrize("layout", [mm.GEMM_NT, mm.GEMM_NN, mm.GEMM_TN])
def test_gemm_bf16_epilogues(layout):
    gemm_case(mm.BF16, layout, 520, 776, 200, bias=True, residual=True, seed=1)
    gemm_case(mm.BF16, layout, 520, 776, 200, accumulate=True, seed=2)
    gemm_case(mm.BF16, layout, 520, 776, 200, bias=True, accumulate=True, residual=True, seed=3)


@pytest.mark.parametrize("layout", [mm.GEMM_NT, mm.GEMM_NN, mm.GEMM_TN])
def test_gemm_bf16_many_tiles(layout):
    # more tiles than compute units' worth of one XCD, ragged in every dimension
    gemm_case(mm.BF16, layout, 2056, 2312, 328, seed=4)


def test_gemm_bf16_few_tiles_cut_along_k():
    # 4 output tiles, K = 4104: with scratch the weight-gradient layout is cut into K chunks (the last one ragged)
    assert mm.mmtrain_gemm_workspace_bytes(mm.GEMM_TN, 512, 392) > 0
    gemm_case(mm.BF16, mm.GEMM_TN, 512, 392, 4104, seed=5, workspace=True)
    gemm_case(mm.BF16, mm.GEMM_TN, 512, 392, 4104, accumulate=True, seed=6, workspace=True)


@pytest.mark.parametrize("layout,accumulate", [(mm.GEMM_NN, False), (mm.GEMM_TN, True), (mm.GEMM_TN, False)])
def test_gemm_bf16_last_round_cut_along_k(layout, accumulate):
    # 18 x 16 = 288 tiles on 256 compute units: the 32 tiles of the second round are cut into 8 K chunks (the last
    # one ragged) whose partial products go through scratch; ragged last tile row and column
    M, N, K = 4360, 4040, 4872
    assert mm.mmtrain_gemm_workspace_bytes(layout, M, N) > 0
    gemm_case(mm.BF16, layout, M, N, K, accumulate=accumulate, seed=7, workspace=True)


@pytest.mark.parametrize("layout", [mm.GEMM_NT, mm.GEMM_NN, mm.GEMM_TN])
@pytest.mark.parametrize("M,N,K", [(7, 5, 3), (130, 70, 33), (512, 768, 256), (64, 64, 0)])
def test_gemm_f32(layout, M, N, K):
    gemm_case(mm.F32, layout, M, N, K, bias=True, residual=True, accumulate=(K == 33))


def attn_case(dtype, nh, nkv, d, cu, modes, seed=0, std=1.0):
    rng = np.random.default_rng(seed)
    T = int(cu[-1])
    nq, nk = nh * d, nkv * d
    qkv = wl.round_to(rng.standard_normal((T, nq + 2 * nk)) * std, dtype)
    d_o = wl.round_to(rng.standard_normal((T, nq)), dtype)
    q = qkv[:, :nq].reshape(T, nh, d).astype(np.float64)
    k = qkv[:, nq:nq + nk].reshape(T, nkv, d).astype(np.float64)
    v = qkv[:, nq + nk:].reshape(T, nkv, d).astype(np.float64)
    scale = 1.0 / np.sqrt(d)
    o_ref, lse_ref = orc.attention_fwd(q, k, v, cu, modes, scale)
    desc = mm.make_desc(mm.DECODER, dtype, 64, nh, nkv, d, 64)
    batch = mm.PackedBatch.on_device(cu, modes)
    wsb = mm.mmtrain_attn_workspace_bytes(T, len(cu) - 1, nh)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    dqkv = to_device(qkv, dtype)
    o = torch.zeros((T, nq), dtype=torch_dtype(dtype), device="cuda")
    lse = torch.zeros((nh, T), dtype=torch.float32, device="cuda")
    check(mm.mmtrain_attn_fwd(desc, batch, dqkv, o, lse, ws, wsb), "mmtrain_attn_fwd")
    torch.cuda.synchronize()
    dq, dk, dv = orc.attention_bwd(d_o.reshape(T, nh, d).astype(np.float64), q, k, v, cu, modes, scale)
    # bf16: the bars follow from what bf16 storage alone costs this very case -- the oracle's attention with the
    # probabilities (and dS) rounded where they feed a matrix-core product and every output rounded once
    f32_bars = {k: 2e-5 for k in ("max_err", "floor_err", "l2_err")}
    floor = {"o": None, "dq": None, "dk": None, "dv": None}
    if dtype == mm.BF16:
        R = bf16_storage.bf16_round
        o_e = R(bf16_storage.attention_fwd_rounded(q, k, v, cu, modes, scale))
        dq_e, dk_e, dv_e = bf16_storage.attention_bwd_rounded(d_o.reshape(T, nh, d).astype(np.float64), o_e, q, k, v, cu, modes, scale)
        floor = {"o": parity.errors(o_e, o_ref), "dq": parity.errors(R(dq_e), dq), "dk": parity.errors(R(dk_e), dk),
                 "dv": parity.errors(R(dv_e), dv)}
    assert_parity("o", to_host(o), o_ref.reshape(T, nq), dtype, None if dtype == mm.BF16 else f32_bars, floor["o"])
    assert np.max(np.abs(lse.cpu().numpy() - lse_ref)) < (2e-2 if dtype == mm.BF16 else 1e-4)
    # backward from the oracle's view of the stored (rounded) output
    d_qkv = torch.zeros_like(dqkv)
    check(mm.mmtrain_attn_bwd(desc, batch, dqkv, o, lse, to_device(d_o, dtype), d_qkv, ws, wsb), "mmtrain_attn_bwd")
    torch.cuda.synchronize()
    got = to_host(d_qkv)
    assert_parity("dq", got[:, :nq], dq.reshape(T, nq), dtype, floor=floor["dq"])
    assert_parity("dk", got[:, nq:nq + nk], dk.reshape(T, nk), dtype, floor=floor["dk"])
    assert_parity("dv", got[:, nq + nk:], dv.reshape(T, nk), dtype, floor=floor["dv"])


RAGGED_CU = np.array([0, 1, 1, 70, 199, 200, 457, 640], dtype=np.int32)   # length-1, empty, mid-tile boundaries
RAGGED_MODES = np.array([0, 1, 1, 0, 1, 0, 1], dtype=np.uint8)


@pytest.mark.parametrize("dtype", [mm.F32, mm.BF16])
@pytest.mark.parametrize("nh,nkv,d", [(4, 4, 64), (4, 2, 128), (8, 1, 64)])
def test_attention_ragged(dtype, nh, nkv, d):
    attn_case(dtype, nh, nkv, d, RAGGED_CU, RAGGED_MODES, std=1.0)


@pytest.mark.parametrize("mode", [0, 1])
def test_attention_one_long_segment(mode):
    attn_case(mm.BF16, 2, 1, 128, np.array([0, 1100], dtype=np.int32), np.array([mode], dtype=np.uint8), seed=3)
    attn_case(mm.BF16, 2, 2, 64, np.array([0, 777], dtype=np.int32), np.array([mode], dtype=np.uint8), seed=4)


@pytest.mark.parametrize("nh,nkv,d", [(4, 4, 80), (4, 2, 80), (2, 2, 96), (4, 1, 32)])
def test_attention_padded_head_dim(nh, nkv, d):
    # head dimensions that are not a native tile width run zero-padded in LDS and registers (80 = ViT-Huge)
    attn_case(mm.BF16, nh, nkv, d, RAGGED_CU, RAGGED_MODES, std=1.0, seed=7)


def test_attention_many_segment_boundaries_wide_head():
    # 128-wide heads take the dK/dV kernel that looks one block ahead: segment boundaries inside key tiles make its
    # wavefronts start and stop at different steps and restart per query head of the group (4 heads per K/V head);
    # segments shorter than one step, a bidirectional segment spanning several key tiles, a ragged end
    rng = np.random.default_rng(11)
    lens = [3, 61, 130, 7, 320, 64, 1, 65, 511, 40, 200, 129]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    modes = rng.integers(0, 2, len(lens)).astype(np.uint8)
    modes[4], modes[8] = 1, 0                                   # the 320-token one bidirectional, the 511-token one causal
    attn_case(mm.BF16, 8, 2, 128, cu, modes, std=1.0, seed=12)


def test_attention_more_tiles_than_the_order_tables_hold():
    # above 16384 tokens a pack has more query / key tiles than the heaviest-first dispatch tables hold (64 / 128
    # entries): the kernels then take their tiles in index order.  Two segments of 8320 tokens, causal and bidirectional.
    cu = np.array([0, 8320, 16640], dtype=np.int32)
    attn_case(mm.BF16, 1, 1, 64, cu, np.array([0, 1], dtype=np.uint8), seed=13)


def test_attention_busy_counters_leave_results_unchanged():
    """The per-compute-unit busy counters (a measurement aid) change nothing in the outputs, and every workgroup's time
    lands in some compute unit's entry."""
    rng = np.random.default_rng(11)
    cu = np.array([0, 300, 301, 1500, 2048], dtype=np.int32)
    modes = np.array([0, 1, 0, 1], dtype=np.uint8)
    T, nh, nkv, d = 2048, 4, 2, 128
    nq, nk = nh * d, nkv * d
    dqkv = to_device(wl.round_to(rng.standard_normal((T, nq + 2 * nk)), mm.BF16), mm.BF16)
    dd_o = to_device(wl.round_to(rng.standard_normal((T, nq)), mm.BF16), mm.BF16)
    desc = mm.make_desc(mm.DECODER, mm.BF16, 64, nh, nkv, d, 64)
    batch = mm.PackedBatch.on_device(cu, modes)
    wsb = mm.mmtrain_attn_workspace_bytes(T, len(cu) - 1, nh)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")

    def run():
        o = torch.zeros((T, nq), dtype=torch.bfloat16, device="cuda")
        lse = torch.zeros((nh, T), dtype=torch.float32, device="cuda")
        d_qkv = torch.zeros_like(dqkv)
        check(mm.mmtrain_attn_fwd(desc, batch, dqkv, o, lse, ws, wsb), "mmtrain_attn_fwd")
        check(mm.mmtrain_attn_bwd(desc, batch, dqkv, o, lse, dd_o, d_qkv, ws, wsb), "mmtrain_attn_bwd")
        torch.cuda.synchronize()
        return o, lse, d_qkv

    plain = run()
    busy = torch.zeros((3, 1024), dtype=torch.int64, device="cuda")
    mm.mmtrain_profile_attn_busy(busy)
    try:
        counted = run()
    finally:
        mm.mmtrain_profile_attn_busy(None)
    for a, b in zip(plain, counted):
        assert torch.equal(a, b)
    rows = busy.cpu().numpy()
    for r in rows:
        used = r[r != 0]
        assert 1 <= used.size <= 256
        assert (used > 0).all() and (used < 100_000_000).all()      # between one tick and a second, at 100 MHz
