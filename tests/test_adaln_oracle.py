"""Pins of the normalised AdaLN modulation oracle to things other than itself: finite differences of the plain
definition, torch's own rms_norm under forward- and reverse-mode autodiff, and special cases.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import adaln_oracle as orc


def rnd(seed, *shape, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def case(seed, B, T, C):
    return (rnd(seed, B, T, C), rnd(seed + 1, B, T, C, scale=0.6), rnd(seed + 2, B, C), rnd(seed + 3, B, C, scale=0.5),
            rnd(seed + 4, B, C), rnd(seed + 5, B, C, scale=0.5), rnd(seed + 6, B, T, C), rnd(seed + 7, B, T, C))


def plain(x, a, b, eps):
    """RMSNorm^-(x) o RMSNorm^-(a) + RMSNorm^-(b), written out (Sec. "Semi-Lipschitz control")."""
    n = lambda v: v / np.sqrt(np.mean(v * v, axis=-1, keepdims=True) + eps)
    return n(x) * n(a)[:, None, :] + n(b)[:, None, :]


@pytest.mark.parametrize("B,T,C", [(1, 1, 2), (2, 3, 5), (2, 4, 24)])
def test_tangent_is_directional_derivative(B, T, C):
    x, tx, a, ta, b, tb, _, _ = case(10, B, T, C)
    eps, h = 1e-4, 1e-5
    fd = (plain(x + h * tx, a + h * ta, b + h * tb, eps) - plain(x - h * tx, a - h * ta, b - h * tb, eps)) / (2 * h)
    y, ty = orc.adaln_jvp_fwd(x, tx, a, ta, b, tb, eps)
    assert np.allclose(y, plain(x, a, b, eps), rtol=1e-13, atol=1e-13)
    assert np.allclose(ty, fd, rtol=1e-7, atol=1e-8)


def loss(p, eps, gy, gty, h=1e-5):
    x, tx, a, ta, b, tb = p
    y = plain(x, a, b, eps)
    ty = (plain(x + h * tx, a + h * ta, b + h * tb, eps) - plain(x - h * tx, a - h * ta, b - h * tb, eps)) / (2 * h)
    return float(np.sum(gy * y) + np.sum(gty * ty))


@pytest.mark.parametrize("B,T,C", [(1, 1, 2), (2, 3, 4), (1, 5, 6)])
def test_every_gradient_entry_by_finite_differences(B, T, C):
    x, tx, a, ta, b, tb, gy, gty = case(20, B, T, C)
    eps, h = 1e-3, 1e-4
    grads = orc.adaln_jvp_bwd(x, tx, a, ta, b, tb, eps, gy, gty)
    params = [x, tx, a, ta, b, tb]
    for k, (arr, grad) in enumerate(zip(params, grads)):
        for idx in np.ndindex(arr.shape):
            p = [v.copy() for v in params]
            p[k][idx] += h
            up = loss(p, eps, gy, gty)
            p[k][idx] -= 2 * h
            dn = loss(p, eps, gy, gty)
            fd = (up - dn) / (2 * h)
            assert abs(fd - grad[idx]) <= 3e-5 * max(1.0, abs(grad[idx])), (k, idx, fd, grad[idx])


def test_against_torch_rms_norm_jvp_and_autograd():
    B, T, C, eps = 2, 5, 16, 1e-5
    vals = case(30, B, T, C)
    T64 = lambda v: torch.tensor(v, dtype=torch.float64)
    x, tx, a, ta, b, tb = (T64(v).requires_grad_(True) for v in vals[:6])
    n = lambda v: torch.nn.functional.rms_norm(v, (C,), eps=eps)
    f = lambda xx, aa, bb: n(xx) * n(aa)[:, None, :] + n(bb)[:, None, :]
    y, ty = torch.func.jvp(f, (x, a, b), (tx, ta, tb))
    oy, oty = orc.adaln_jvp_fwd(*vals[:6], eps)
    assert np.allclose(oy, y.detach().numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(oty, ty.detach().numpy(), rtol=1e-11, atol=1e-12)
    ((y * T64(vals[6])).sum() + (ty * T64(vals[7])).sum()).backward()
    got = orc.adaln_jvp_bwd(*vals[:6], eps, vals[6], vals[7])
    for g, t in zip(got, (x, tx, a, ta, b, tb)):
        assert np.allclose(g, t.grad.numpy(), rtol=1e-10, atol=1e-11)


def test_constant_scale_and_zero_tangents():
    B, T, C = 2, 3, 8
    x, tx, a, ta, b, tb, gy, gty = case(40, B, T, C)
    # a constant vector normalises to ones (eps = 0): the modulation is then RMSNorm^-(x) + RMSNorm^-(b)
    y, _ = orc.adaln_jvp_fwd(x, tx, np.full((B, C), 3.0), ta, b, tb, 0.0)
    n = lambda v: v / np.sqrt(np.mean(v * v, axis=-1, keepdims=True))
    assert np.allclose(y, n(x) + n(b)[:, None, :], rtol=1e-13)
    _, z = orc.adaln_jvp_fwd(x, np.zeros_like(x), a, np.zeros_like(a), b, np.zeros_like(b), 1e-3)
    assert np.all(z == 0.0)
    # tangents enter linearly
    _, t1 = orc.adaln_jvp_fwd(x, tx, a, ta, b, tb, 1e-3)
    _, t2 = orc.adaln_jvp_fwd(x, 2 * tx, a, 2 * ta, b, 2 * tb, 1e-3)
    assert np.allclose(t2, 2 * t1, rtol=1e-12, atol=1e-13)


def test_modulation_gradients_sum_over_the_tokens_of_a_batch_element():
    B, T, C = 2, 4, 6
    x, tx, a, ta, b, tb, gy, gty = case(50, B, T, C)
    full = orc.adaln_jvp_bwd(x, tx, a, ta, b, tb, 1e-4, gy, gty)
    # the loss is a sum over tokens, so the gradients of a and b are sums of one-token gradients
    for bb in range(B):
        acc = [np.zeros(C) for _ in range(4)]
        for t in range(T):
            one = orc.adaln_jvp_bwd(x[bb:bb + 1, t:t + 1], tx[bb:bb + 1, t:t + 1], a[bb:bb + 1], ta[bb:bb + 1],
                                    b[bb:bb + 1], tb[bb:bb + 1], 1e-4, gy[bb:bb + 1, t:t + 1], gty[bb:bb + 1, t:t + 1])
            assert np.allclose(one[0][0, 0], full[0][bb, t], rtol=1e-12, atol=1e-13)
            assert np.allclose(one[1][0, 0], full[1][bb, t], rtol=1e-12, atol=1e-13)
            for k in range(4):
                acc[k] += one[2 + k][0]
        for k in range(4):
            assert np.allclose(acc[k], full[2 + k][bb], rtol=1e-12, atol=1e-13)
