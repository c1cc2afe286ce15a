"""Pins of the oracle's optimizer step (SGD with Nesterov momentum, Appendix A table
"Hyperparameters"; update rule of Section 3) against things other than itself: the library
optimizer, closed forms of the recurrence, and the special cases that reduce to plain SGD."""
import numpy as np
import pytest
import torch

from oracle import accordion_oracle as orc

F32 = np.float32
EPS = float(np.finfo(np.float32).eps)


def _run_oracle(w0, ds, lr, mu, wd):
    w, v = w0.copy(), np.zeros_like(w0)
    for d in ds:
        w, v = orc.nesterov_update(w, v, d, lr, mu, wd)
    return w, v


@pytest.mark.parametrize("wd", [0.0, 5e-4])
@pytest.mark.parametrize("mu", [0.9, 0.5])
def test_matches_the_library_optimizer(mu, wd):
    """torch.optim.SGD(nesterov=True) in fp64 is the reference recurrence; the oracle's fp32
    steps stay within a few roundings per step of it."""
    rng = np.random.default_rng(3)
    n, steps, lr = 257, 12, 0.4
    w0 = rng.standard_normal(n).astype(F32)
    ds = [rng.standard_normal(n).astype(F32) for _ in range(steps)]
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, nesterov=True, weight_decay=wd)
    for d in ds:
        p.grad = torch.tensor(d, dtype=torch.float64)
        opt.step()
    w, v = _run_oracle(w0, ds, lr, mu, wd)
    ref_w = p.detach().numpy()
    ref_v = opt.state[p]["momentum_buffer"].numpy()
    scale = np.abs(ref_w) + lr * 10.0 * np.abs(ref_v) + 1.0
    assert np.all(np.abs(w - ref_w) <= 8 * steps * EPS * scale)
    assert np.all(np.abs(v - ref_v) <= 8 * steps * EPS * (np.abs(ref_v) + 1.0))


def test_library_optimizer_in_fp32_agrees_too():
    """Same comparison against the library's own fp32 arithmetic (its fused multiply-adds may
    round differently, hence a tolerance of a few ulps rather than equality)."""
    rng = np.random.default_rng(4)
    n, lr, mu = 100, 0.1, 0.9
    w0 = rng.standard_normal(n).astype(F32)
    ds = [rng.standard_normal(n).astype(F32) for _ in range(5)]
    p = torch.nn.Parameter(torch.tensor(w0))
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, nesterov=True)
    for d in ds:
        p.grad = torch.tensor(d)
        opt.step()
    w, v = _run_oracle(w0, ds, lr, mu, 0.0)
    assert np.allclose(w, p.detach().numpy(), rtol=0, atol=32 * EPS * 4.0)
    assert np.allclose(v, opt.state[p]["momentum_buffer"].numpy(), rtol=0, atol=32 * EPS * 10.0)


def test_constant_gradient_closed_form():
    """With a constant gradient d and v_0 = 0: v_n = d (1 - mu^n)/(1 - mu) and
    w_n = w_0 - lr * sum_{k=1..n} (d + mu v_k)."""
    mu, lr, n = 0.9, 0.05, 40
    d = np.array([1.0, -2.0, 0.5, 0.0], dtype=F32)
    w0 = np.array([0.0, 1.0, -1.0, 3.0], dtype=F32)
    w, v = _run_oracle(w0, [d] * n, lr, mu, 0.0)
    d64, w64 = d.astype(np.float64), w0.astype(np.float64)
    v_n = d64 * (1 - mu ** n) / (1 - mu)
    look_sum = sum(1 + mu * (1 - mu ** k) / (1 - mu) for k in range(1, n + 1))
    w_n = w64 - lr * d64 * look_sum
    assert np.allclose(v, v_n, rtol=1e-5, atol=0)
    assert np.allclose(w, w_n, rtol=1e-5, atol=1e-6)
    assert w[3] == F32(3.0) and v[3] == F32(0.0)          # a zero gradient moves nothing


def test_without_momentum_it_is_the_plain_update_rule():
    """mu = 0: w_{k+1} = w_k - gamma d exactly, one product and one difference in fp32."""
    rng = np.random.default_rng(5)
    w0 = rng.standard_normal(1000).astype(F32)
    d = rng.standard_normal(1000).astype(F32)
    w, v = orc.nesterov_update(w0, np.zeros_like(w0), d, 0.3, 0.0)
    assert np.array_equal(w, (w0 - (F32(0.3) * d).astype(F32)).astype(F32))
    assert np.array_equal(v, d)


def test_first_step_and_look_ahead_factor():
    """From v = 0 the first Nesterov step moves by lr (1 + mu) d, not lr d (heavy ball) and not
    lr mu d; with lr = 0 the weights stay and the velocity still moves."""
    d = np.array([0.5, -0.25], dtype=F32)
    w0 = np.array([1.0, 1.0], dtype=F32)
    w, v = orc.nesterov_update(w0, np.zeros(2, F32), d, 0.5, 0.5)
    assert np.array_equal(v, d)
    assert np.array_equal(w, w0 - F32(0.5) * F32(1.5) * d)          # all exact in binary
    w2, v2 = orc.nesterov_update(w0, v, d, 0.0, 0.5)
    assert np.array_equal(w2, w0) and np.array_equal(v2, F32(1.5) * d)


def test_weight_decay_enters_as_a_gradient_term():
    """lambda w is added to the gradient before the momentum (so it is in v as well)."""
    w0 = np.array([2.0, -4.0], dtype=F32)
    d = np.array([1.0, 1.0], dtype=F32)
    w, v = orc.nesterov_update(w0, np.zeros(2, F32), d, 0.25, 0.5, 0.5)
    dd = d + F32(0.5) * w0                                           # [2, -1]
    assert np.array_equal(v, dd)
    assert np.array_equal(w, w0 - F32(0.25) * F32(1.5) * dd)


def test_step_update_touches_only_layer_elements_and_uses_the_step_mean():
    layers = [(0, 3, 4, 1), (16, 1, 5, 0)]                  # a gap between the layers
    n_flat = 21
    o = orc.AccordionOracle(orc.TOPK, layers, 2, 50, 10, 100)
    o.N = n_flat
    o.e = np.zeros((2, n_flat), F32)
    o.A = np.zeros(n_flat, F32)
    rng = np.random.default_rng(6)
    grads = [rng.standard_normal(n_flat).astype(F32) for _ in range(2)]
    w = rng.standard_normal(n_flat).astype(F32)
    v = rng.standard_normal(n_flat).astype(F32)
    w_before, v_before = w.copy(), v.copy()
    d = o.step_update(grads, w, v, 0.1, 0.9)
    assert np.array_equal(w[12:16], w_before[12:16]) and np.array_equal(v[12:16], v_before[12:16])
    for off, r, c, _ in layers:
        sl = slice(off, off + r * c)
        ew, ev = orc.nesterov_update(w_before[sl], v_before[sl], d[sl], 0.1, 0.9)
        assert np.array_equal(w[sl], ew) and np.array_equal(v[sl], ev)
        assert np.count_nonzero(d[sl]) > 0
