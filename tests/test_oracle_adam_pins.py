"""Pins of the optimizer oracle (oracle/optim.py) against things other than itself: closed forms of Adam's first step
and of a constant gradient (the bias correction), torch's own Adam / AdamW in double precision, scaling and clipping
identities.  Hyperparameters from the paper's appendix: beta2 = 0.999, max grad norm 0.3, lr 2e-4 / 1e-4."""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import optim

LR, B1, B2, EPS = 2e-4, 0.9, 0.999, 1e-8


def _rand(n, seed, sigma=1.0):
    return np.random.Generator(np.random.Philox(key=seed)).standard_normal(n) * sigma


def test_first_step_is_lr_times_sign_with_eps():
    """m0 = v0 = 0, t = 1: m^ = g and v^ = g^2, so p1 = p0 - lr * g / (|g| + eps)."""
    p0, g = _rand(1000, 1), _rand(1000, 2, 1e-3)
    g[:3] = [0.0, 1e-12, -1e-12]                              # at and below eps: the step shrinks to lr * g / eps
    p1, m1, v1 = optim.adam_step(p0, np.zeros(1000), np.zeros(1000), g, 1, LR, B1, B2, EPS)
    np.testing.assert_allclose(p1, p0 - LR * g / (np.abs(g) + EPS), rtol=0, atol=1e-15)
    np.testing.assert_allclose(m1, (1 - B1) * g, rtol=1e-15)
    np.testing.assert_allclose(v1, (1 - B2) * g * g, rtol=1e-13)
    assert p1[0] == p0[0]


def test_constant_gradient_closed_form():
    """A constant gradient: m_t = (1 - beta1^t) g, v_t = (1 - beta2^t) g^2, so every step moves lr * g / (|g| + eps)."""
    p0, g = _rand(64, 3), _rand(64, 4, 0.05)
    p, m, v = p0.copy(), np.zeros(64), np.zeros(64)
    for t in range(1, 41):
        p, m, v = optim.adam_step(p, m, v, g, t, LR, B1, B2, EPS)
        np.testing.assert_allclose(m, (1 - B1 ** t) * g, rtol=1e-12)
        np.testing.assert_allclose(v, (1 - B2 ** t) * g * g, rtol=1e-12)
        np.testing.assert_allclose(p, p0 - t * LR * g / (np.abs(g) + EPS), rtol=0, atol=1e-13)


@pytest.mark.parametrize("wd", [0.0, 0.01])
def test_against_torch_adam_in_double(wd):
    """The library's optimizer on the same sequence of gradients (AdamW is the decoupled decay)."""
    n, steps = 257, 12
    p0 = _rand(n, 10)
    tp = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = (torch.optim.AdamW if wd else torch.optim.Adam)([tp], lr=LR, betas=(B1, B2), eps=EPS, weight_decay=wd)
    p, m, v = p0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, steps + 1):
        g = _rand(n, 100 + t, 0.02 * t)
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        p, m, v = optim.adam_step(p, m, v, g, t, LR, B1, B2, EPS, weight_decay=wd)
        np.testing.assert_allclose(p, tp.detach().numpy(), rtol=0, atol=1e-14)
    st = opt.state[tp]
    np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-300)
    assert np.abs(p - p0).max() > 5 * LR                      # the parameters did move


def test_coefficient_scales_the_gradient():
    p0, m0, v0, g = _rand(100, 20), _rand(100, 21, 0.01), np.abs(_rand(100, 22, 1e-4)), _rand(100, 23, 0.3)
    a = optim.adam_step(p0, m0, v0, g, 7, LR, coef=0.125)
    b = optim.adam_step(p0, m0, v0, 0.125 * g, 7, LR)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)                   # a power of two: exact


def test_clipping_by_global_norm():
    g = _rand(5000, 30, 0.02)
    sq = optim.sqnorm(g)
    assert sq == pytest.approx(math.fsum(float(x) * float(x) for x in g), rel=1e-14)
    assert optim.sqnorm(np.full(64, 0.5)) == 16.0
    norm = math.sqrt(sq)
    assert norm > 0.3
    c = optim.grad_coefficient(sq, 0.3)
    assert np.linalg.norm(c * g) == pytest.approx(0.3, rel=1e-12)
    assert optim.grad_coefficient(sq, 2 * norm) == 1.0        # below the limit: untouched
    assert optim.grad_coefficient(sq, 0.0, 0.25) == 0.25      # no limit
    # accumulated over 16 micro-batches: the norm that counts is that of the averaged gradient
    c16 = optim.grad_coefficient(256.0 * sq, 0.3, 1.0 / 16)
    assert c16 == pytest.approx(c / 16, rel=1e-14)
    assert optim.grad_coefficient(0.0, 0.3) == 1.0


def test_single_precision_steps_follow_the_definition():
    """The fp32 mode takes the same steps: it stays within a few fp32 roundings of the double-precision result, and the
    bf16 copy of its parameters is a plain round-to-nearest-even of them."""
    n = 4096
    p0 = _rand(n, 40, 0.02).astype(np.float32)
    g = _rand(n, 41, 0.01).astype(np.float32)
    p64, m64, v64 = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    p32, m32, v32 = p0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    for t in range(1, 6):
        p64, m64, v64 = optim.adam_step(p64, m64, v64, g, t, LR)
        p32, m32, v32 = optim.adam_step(p32, m32, v32, g, t, LR, dtype=np.float32)
    assert p32.dtype == np.float32
    np.testing.assert_allclose(m32, m64, rtol=1e-6, atol=1e-30)
    np.testing.assert_allclose(v32, v64, rtol=1e-6, atol=1e-30)
    assert np.abs(p32 - p64).max() <= 5 * 2.0 ** -24 * np.abs(p64).max() + 5 * LR * 4e-7
    bits = np.array([oracle.bf16_rne(x) for x in p32[:256]], dtype=np.uint16)
    tb = torch.from_numpy(p32[:256].copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, tb)
