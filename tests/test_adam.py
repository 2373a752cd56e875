"""The optimizer step: oracle against closed forms and an independent library routine (CPU), C-ABI argument
checks (CPU), and the HIP kernel against the oracle (GPU)."""
import numpy as np
import pytest
import torch

from oracle import adam_oracle as ao
from paper_2408_04275_amd import binding as mm
from paper_2408_04275_amd import workloads as wl


def test_oracle_first_step_moves_by_lr_times_sign():
    # zero state, t = 1: the bias-corrected moments are g and g^2, so the step is lr * g / (|g| + eps)
    g = np.array([3.0, -0.5, 1e-3, -7.0])
    w, m, v = ao.adam_step(np.zeros(4), g, np.zeros(4), np.zeros(4), 0.1, 0.9, 0.999, 1e-12, 0.0, 1.0, 1)
    assert np.allclose(w, -0.1 * np.sign(g), rtol=1e-8)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)


def test_oracle_constant_gradient_walks_in_equal_steps():
    # with a constant gradient the corrected moments stay g and g^2 at every t: w_t = w_0 - t lr sign(g)
    g = np.array([2.0, -4.0])
    w, m, v = np.array([1.0, 1.0]), np.zeros(2), np.zeros(2)
    for t in range(1, 8):
        w, m, v = ao.adam_step(w, g, m, v, 0.01, 0.9, 0.95, 1e-15, 0.0, 1.0, t)
        assert np.allclose(w, 1.0 - t * 0.01 * np.sign(g), rtol=1e-10)


def test_oracle_weight_decay_is_decoupled():
    # zero gradient: only the decay acts, w <- w (1 - lr wd), and the moments stay zero
    w, m, v = ao.adam_step(np.array([2.0, -3.0]), np.zeros(2), np.zeros(2), np.zeros(2), 0.1, 0.9, 0.999, 1e-8, 0.5, 1.0, 3)
    assert np.allclose(w, np.array([2.0, -3.0]) * (1 - 0.05)) and not m.any() and not v.any()


def test_oracle_matches_torch_adamw_over_several_steps():
    rng = np.random.default_rng(0)
    w0 = rng.standard_normal(257)
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.1)
    w, m, v = w0.copy(), np.zeros(257), np.zeros(257)
    for t in range(1, 6):
        g = rng.standard_normal(257) * (10.0 ** rng.integers(-3, 2, size=257))
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m, v = ao.adam_step(w, g, m, v, 3e-3, 0.9, 0.95, 1e-8, 0.1, 1.0, t)
        assert np.allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_oracle_grad_scale_is_a_plain_prefactor():
    rng = np.random.default_rng(1)
    w, g = rng.standard_normal(16), rng.standard_normal(16)
    a = ao.adam_step(w, g, np.zeros(16), np.zeros(16), 1e-2, 0.9, 0.999, 1e-8, 0.01, 0.25, 1)
    b = ao.adam_step(w, 0.25 * g, np.zeros(16), np.zeros(16), 1e-2, 0.9, 0.999, 1e-8, 0.01, 1.0, 1)
    for x, y in zip(a, b):
        assert np.allclose(x, y, rtol=1e-14)


def test_c_abi_rejects_bad_arguments():
    F = 0x1000
    ok = mm.make_adam_desc(1e-3)
    assert mm.mmtrain_adam_step(ok, 0, None, None, None, None, None, mm.BF16, 0) == mm.OK
    assert mm.mmtrain_adam_step(None, 4, F, F, F, F, F, mm.BF16, 0) == mm.ERR_INVALID_ARG
    assert mm.mmtrain_adam_step(ok, -1, F, F, F, F, F, mm.BF16, 0) == mm.ERR_INVALID_ARG
    assert mm.mmtrain_adam_step(ok, 4, None, F, F, F, F, mm.BF16, 0) == mm.ERR_INVALID_ARG
    assert mm.mmtrain_adam_step(ok, 4, F + 4, F, F, F, F, mm.BF16, 0) == mm.ERR_INVALID_ARG
    assert mm.mmtrain_adam_step(ok, 4, F, F, F, F, F, 7, 0) == mm.ERR_INVALID_ARG
    for bad in (dict(lr=-1.0), dict(lr=1e-3, beta1=1.0), dict(lr=1e-3, beta2=-0.1), dict(lr=1e-3, eps=0.0),
                dict(lr=1e-3, weight_decay=-1.0), dict(lr=1e-3, step=0), dict(lr=float("nan"))):
        assert mm.mmtrain_adam_step(mm.make_adam_desc(**bad), 4, F, F, F, F, F, mm.BF16, 0) == mm.ERR_INVALID_ARG
    d = mm.make_adam_desc(1e-3)
    d.struct_size = 8
    assert mm.mmtrain_adam_step(d, 4, F, F, F, F, F, mm.BF16, 0) == mm.ERR_INVALID_ARG


@pytest.mark.gpu
@pytest.mark.parametrize("n", [1, 5, 1024, 4099, 1 << 20])
@pytest.mark.parametrize("param_dtype", [mm.BF16, mm.F32])
def test_gpu_adam_matches_the_oracle(n, param_dtype):
    rng = np.random.default_rng(n)
    w = rng.standard_normal(n).astype(np.float32)
    m = (rng.standard_normal(n) * 0.1).astype(np.float32)
    v = (rng.random(n) * 0.01).astype(np.float32)
    dev = lambda a: torch.tensor(a, device="cuda")
    dw, dm, dv = dev(w), dev(m), dev(v)
    out = torch.zeros(n, device="cuda", dtype=torch.bfloat16 if param_dtype == mm.BF16 else torch.float32)
    rw, rm, rv = w.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
    # the description carries fp32 hyperparameters: the oracle gets the same values (0.999 as fp32 is 0.99900001,
    # which changes 1 - beta2 by 1.3e-5)
    lr, b1, b2, eps, wd, gs = (float(np.float32(x)) for x in (2e-3, 0.9, 0.999, 1e-8, 0.1, 0.5))
    for t in (7, 8, 9):
        g = (rng.standard_normal(n) * (10.0 ** rng.integers(-4, 3, size=n))).astype(np.float32)
        dg = dev(g)
        desc = mm.make_adam_desc(2e-3, 0.9, 0.999, 1e-8, 0.1, 0.5, t, zero_grad=(t == 9))
        assert mm.mmtrain_adam_step(desc, n, dw, dg, dm, dv, out, param_dtype) == mm.OK
        rw, rm, rv = ao.adam_step(rw, g, rm, rv, lr, b1, b2, eps, wd, gs, t)
        torch.cuda.synchronize()
        assert np.array_equal(dg.cpu().numpy(), g if t != 9 else np.zeros_like(g))
    # fp32 arithmetic against fp64: a few ulp per step on w, m, v
    # (an element whose second moment is tiny takes a step of many times lr; its error scales with the step)
    assert np.allclose(dw.cpu().numpy(), rw, rtol=4e-6, atol=2e-6)
    # (a moment that nearly cancels keeps the absolute error of its two terms)
    assert np.allclose(dm.cpu().numpy(), rm, rtol=2e-6, atol=1e-6 * np.abs(rm).max())
    assert np.allclose(dv.cpu().numpy(), rv, rtol=2e-6, atol=1e-6 * np.abs(rv).max())
    # the working copy is the fp32 master rounded once
    want = wl.round_bf16(dw.cpu().numpy()) if param_dtype == mm.BF16 else dw.cpu().numpy()
    assert np.array_equal(out.float().cpu().numpy(), want)
