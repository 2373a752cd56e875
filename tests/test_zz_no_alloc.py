"""mmtrain_attn_bwd_noalloc (attention backward with its scratch in a fixed device array inside the library) against
mmtrain_attn_bwd on the same inputs, through the C ABI: two calls in a row, the second with a smaller input, so that
what the first call left in the shared array cannot leak into the second; and the size limits, which are checked on
the host before anything is enqueued."""
import numpy as np
import pytest
import torch

from oracle import layer_oracle as orc
from paper_2408_04275_amd import binding as mm
from paper_2408_04275_amd import workloads as wl
from paper_2408_04275_amd.harness import check, to_device, to_host
from util import assert_parity, say


def attention_inputs(nh, nkv, d, cu, seed):
    rng = np.random.default_rng(seed)
    T = int(cu[-1])
    qkv = wl.round_to(rng.standard_normal((T, (nh + 2 * nkv) * d)), mm.BF16)
    d_o = wl.round_to(rng.standard_normal((T, nh * d)), mm.BF16)
    return qkv, d_o


@pytest.mark.gpu
def test_no_alloc_attention_backward_matches_the_workspace_entry_point():
    cases = [(8, 2, 128, np.array([0, 3, 64, 194, 514, 578, 579, 644, 1155, 1195, 1395, 1524], dtype=np.int32), 21),
             (4, 4, 64, np.array([0, 1, 1, 70, 199, 200, 457, 640], dtype=np.int32), 22)]      # the second one smaller
    for nh, nkv, d, cu, seed in cases:
        S, T = len(cu) - 1, int(cu[-1])
        modes = np.random.default_rng(seed).integers(0, 2, S).astype(np.uint8)
        qkv, d_o = attention_inputs(nh, nkv, d, cu, seed)
        desc = mm.make_desc(mm.DECODER, mm.BF16, 64, nh, nkv, d, 64)
        batch = mm.PackedBatch.on_device(cu, modes)
        wsb = mm.mmtrain_attn_workspace_bytes(T, S, nh)
        ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        dqkv, dd_o = to_device(qkv, mm.BF16), to_device(d_o, mm.BF16)
        o = torch.zeros((T, nh * d), dtype=torch.bfloat16, device="cuda")
        lse = torch.zeros((nh, T), dtype=torch.float32, device="cuda")
        check(mm.mmtrain_attn_fwd(desc, batch, dqkv, o, lse, ws, wsb), "mmtrain_attn_fwd")
        want = torch.full_like(dqkv, float("nan"))
        got = torch.full_like(dqkv, float("nan"))
        say(f"no-alloc attention backward: T={T} heads={nh}/{nkv}x{d} segments={np.diff(cu).tolist()}")
        check(mm.mmtrain_attn_bwd(desc, batch, dqkv, o, lse, dd_o, want, ws, wsb), "mmtrain_attn_bwd")
        check(mm.mmtrain_attn_bwd_noalloc(desc, batch, dqkv, o, lse, dd_o, got), "mmtrain_attn_bwd_noalloc")
        torch.cuda.synchronize()
        assert torch.equal(got, want)                              # same kernels, same order of summation: same bits
        # and both are the oracle's gradient, to the operator-level bars
        nq, nk = nh * d, nkv * d
        q = qkv[:, :nq].reshape(T, nh, d).astype(np.float64)
        k = qkv[:, nq:nq + nk].reshape(T, nkv, d).astype(np.float64)
        v = qkv[:, nq + nk:].reshape(T, nkv, d).astype(np.float64)
        dq, dk, dv = orc.attention_bwd(d_o.reshape(T, nh, d).astype(np.float64), q, k, v, cu, modes, 1.0 / np.sqrt(d))
        g = to_host(got)
        assert_parity("dq", g[:, :nq], dq.reshape(T, nq), mm.BF16)
        assert_parity("dk", g[:, nq:nq + nk], dk.reshape(T, nk), mm.BF16)
        assert_parity("dv", g[:, nq + nk:], dv.reshape(T, nk), mm.BF16)


def test_no_alloc_limits_are_checked_on_the_host():
    # no GPU needed: the size check comes before any device pointer is looked at
    def call(T, nh):
        cu = np.array([0, T], dtype=np.int32)
        batch = mm.PackedBatch(cu, None, mm.MASK_CAUSAL, cu_dev=1 << 20)         # never dereferenced
        desc = mm.make_desc(mm.DECODER, mm.BF16, 64, nh, nh, 64, 64)
        return mm.mmtrain_attn_bwd_noalloc(desc, batch, None, None, None, None, None, 0)
    assert call(mm.NOALLOC_MAX_TOKENS + 1, 1) == mm.ERR_TOO_LARGE
    assert call(mm.NOALLOC_MAX_TOKENS, 65) == mm.ERR_TOO_LARGE
    assert call(8192, 129) == mm.ERR_TOO_LARGE
    assert call(0, 4) == mm.OK                                                    # an empty pack is a no-op
    assert call(256, 4) == mm.ERR_INVALID_ARG                                     # within the limits: NULL tensors are rejected next
    assert "static scratch" in mm.mmtrain_status_string(mm.ERR_TOO_LARGE)
