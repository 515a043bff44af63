"""Optimizer step of the LoRA parameters (qlora_adam_step, qlora_grad_sqnorm) against oracle/optim.py.

The kernel computes in fp32 with every operation rounded separately, so against the oracle's fp32 mode (the same steps
in numpy float32) parameters, moments and the bf16 copy are compared BIT FOR BIT; against the double-precision
definition the bound is a few fp32 roundings.  The clipped path goes through a double-precision sum whose order of
additions is not fixed, so there the coefficient may differ in its last fp32 bit and the comparison uses the bound."""
import numpy as np
import pytest
import torch

import oracle
from oracle import optim
import paper_2305_14314_amd as q
from gpu_util import host_bits

pytestmark = pytest.mark.gpu

LR, B1, B2, EPS = 1e-4, 0.9, 0.999, 1e-8                      # 65B row of the hyperparameter table


def _rand(n, seed, sigma):
    return (np.random.Generator(np.random.Philox(key=seed)).standard_normal(n) * sigma).astype(np.float32)


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _lora_block_sizes(d=8192, ffn=22016, r=64):
    """Parameter count of the adapters of one 65B-shaped decoder block: L1 (h x r) and L2 (r x o) of its 7 linears."""
    shapes = [(d, d)] * 4 + [(d, ffn)] * 2 + [(ffn, d)]
    return sum(h * r + r * o for h, o in shapes)


@pytest.mark.parametrize("n", [0, 1, 3, 4, 7, 1024, 8192 * 64 + 5, _lora_block_sizes()])
@pytest.mark.parametrize("wd", [0.0, 0.01])
def test_adam_steps_bit_exact(n, wd):
    if n > 10 ** 6 and wd:
        pytest.skip("one full-size case is enough")
    print(f"adam: n {n} wd {wd}", flush=True)
    p0 = _rand(n, 1, 0.02)
    p, m, v = p0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    dp, dm, dv = _dev(p), _dev(m), _dev(v)
    dpb = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    steps = 2 if n > 10 ** 6 else 4
    for t in range(1, steps + 1):
        g = _rand(n, 10 + t, 0.003 * t)
        if n >= 1024:
            g[:8] = [0.0, 1e-12, -1e-12, 1e-20, -3e-23, 1e-30, 1.0, -1.0]   # below eps, squares that underflow, large
        dg = _dev(g)
        scale = 1.0 / 16                                      # a sum over 16 micro-batches
        q.qlora_adam_step(dp, dm, dv, dg, t, LR, B1, B2, EPS, weight_decay=wd, grad_scale=scale, param_bf16=dpb,
                          zero_grad=(t % 2 == 0))
        p, m, v = optim.adam_step(p, m, v, g, t, LR, B1, B2, EPS, weight_decay=wd, coef=scale, dtype=np.float32)
        torch.cuda.synchronize()
        for name, got, ref in (("m", dm, m), ("v", dv, v), ("p", dp, p)):
            gh = got.cpu().numpy()
            bad = np.flatnonzero(gh.view(np.uint32) != ref.view(np.uint32))
            assert bad.size == 0, (name, t, bad[:5], gh[bad[:5]], ref[bad[:5]])
        if n:
            tb = torch.from_numpy(p.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
            np.testing.assert_array_equal(host_bits(dpb), tb)
            samp = np.linspace(0, n - 1, min(n, 64)).astype(np.int64)
            assert [oracle.bf16_rne(float(p[i])) for i in samp] == [int(tb[i]) for i in samp]
        gz = dg.cpu().numpy()
        if t % 2 == 0:
            assert not gz.any()                                # consumed
        else:
            np.testing.assert_array_equal(gz, g)               # left alone
    if n >= 1024:
        assert np.abs(p - p0).max() > LR                       # it moved


def test_adam_against_the_double_precision_definition():
    n = 8192 * 64
    p0, g = _rand(n, 3, 0.02), _rand(n, 4, 0.01)
    dp, dm, dv, dg = _dev(p0), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda"), _dev(g)
    p, m, v = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t in range(1, 6):
        q.qlora_adam_step(dp, dm, dv, dg, t, LR, B1, B2, EPS)
        p, m, v = optim.adam_step(p, m, v, g, t, LR, B1, B2, EPS)
    torch.cuda.synchronize()
    np.testing.assert_allclose(dm.cpu().numpy(), m, rtol=1e-6, atol=1e-30)
    np.testing.assert_allclose(dv.cpu().numpy(), v, rtol=1e-6, atol=1e-30)
    # per step: one rounding of p (2^-24 |p|) and a relative error of a few 1e-7 on a step of at most lr
    assert np.abs(dp.cpu().numpy() - p).max() <= 5 * (2.0 ** -24 * np.abs(p).max() + LR * 1e-6)


@pytest.mark.parametrize("n", [5, 4096, 3 * 8192 * 64 + 1])
def test_sqnorm(n):
    g = _rand(n, 7, 0.05)
    acc = torch.zeros(1, dtype=torch.float64, device="cuda")
    q.qlora_grad_sqnorm(_dev(g), acc)
    q.qlora_grad_sqnorm(_dev(g[: n // 2]), acc)                # accumulates over buffers
    want = optim.sqnorm(g) + optim.sqnorm(g[: n // 2])
    assert acc.item() == pytest.approx(want, rel=1e-12)


def test_adam_with_clipping_to_the_papers_norm():
    """Two parameter buffers, one global norm; max grad norm 0.3 (hyperparameter appendix)."""
    na, nb = 8192 * 64, 64 * 22016
    ga, gb = _rand(na, 20, 0.01), _rand(nb, 21, 0.02)
    sq = optim.sqnorm(ga) + optim.sqnorm(gb)
    scale = 0.5
    coef = optim.grad_coefficient(sq, 0.3, scale)
    assert coef < scale                                        # the limit bites
    acc = torch.zeros(1, dtype=torch.float64, device="cuda")
    bufs = []
    for g in (ga, gb):
        dg = _dev(g)
        q.qlora_grad_sqnorm(dg, acc)
        bufs.append(dg)
    for g, dg, seed in ((ga, bufs[0], 30), (gb, bufs[1], 31)):
        n = g.size
        p0 = _rand(n, seed, 0.02)
        dp, dm, dv = _dev(p0), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
        q.qlora_adam_step(dp, dm, dv, dg, 1, LR, B1, B2, EPS, grad_scale=scale, max_grad_norm=0.3, sqnorm=acc)
        p, m, v = optim.adam_step(p0, np.zeros(n), np.zeros(n), g, 1, LR, B1, B2, EPS, coef=coef)
        torch.cuda.synchronize()
        np.testing.assert_allclose(dm.cpu().numpy(), m, rtol=1e-6, atol=1e-30)
        np.testing.assert_allclose(dv.cpu().numpy(), v, rtol=1e-6, atol=1e-30)
        assert np.abs(dp.cpu().numpy() - p).max() <= 2.0 ** -24 * np.abs(p).max() + LR * 1e-6
    # without a limit the same call leaves the gradient at grad_scale
    n = 4096
    g, p0 = _rand(n, 40, 1.0), _rand(n, 41, 0.02)
    dp, dm, dv = _dev(p0), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    q.qlora_adam_step(dp, dm, dv, _dev(g), 1, LR, B1, B2, EPS, grad_scale=scale, max_grad_norm=0.0, sqnorm=acc)
    _, m, _ = optim.adam_step(p0, np.zeros(n, np.float32), np.zeros(n, np.float32), g, 1, LR, B1, B2, EPS, coef=scale,
                              dtype=np.float32)
    np.testing.assert_array_equal(dm.cpu().numpy(), m)


def test_adam_argument_errors_launch_nothing():
    L = q.lib()
    t = torch.zeros(64, device="cuda")
    cfg = q.qlora_adam_config(1e-4, 0.9, 0.999, 1e-8, 0.0, 1.0, 0.0, 0, 0, 0)      # step 0
    import ctypes
    p = ctypes.c_void_p(t.data_ptr())
    assert L.qlora_adam_step(p, p, p, p, None, 64, ctypes.byref(cfg), None, None) == -2
    cfg.step = 1
    assert L.qlora_adam_step(None, p, p, p, None, 64, ctypes.byref(cfg), None, None) == -1
    assert L.qlora_adam_step(ctypes.c_void_p(t.data_ptr() + 4), p, p, p, None, 64, ctypes.byref(cfg), None, None) == -5
    cfg.beta2 = 1.0
    assert L.qlora_adam_step(p, p, p, p, None, 64, ctypes.byref(cfg), None, None) == -3
    torch.cuda.synchronize()
    assert not t.cpu().numpy().any()
