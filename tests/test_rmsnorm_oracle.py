"""Pins of the RMSNorm (QK-norm) oracle to things other than itself: the Jacobian the paper prints
(App. "Lipschitzness of RMSNorm"), finite differences, torch's own rms_norm under forward- and
reverse-mode autodiff, a hand-derived closed form, and invariants.  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import rmsnorm_oracle as orc


def rnd(seed, *shape, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def case(seed, rows, d):
    return (rnd(seed, rows, d), rnd(seed + 1, rows, d, scale=0.7), 1.0 + 0.3 * rnd(seed + 2, d),
            rnd(seed + 3, rows, d), rnd(seed + 4, rows, d))


# ---------------------------------------------------------------------------- 1. what the paper prints
@pytest.mark.parametrize("d", [1, 2, 7, 72])
def test_tangent_is_the_printed_jacobian_times_the_input_tangent(d):
    """d RMSNorm(x)_i / d x_j = delta_ij / RMS - x_i x_j / (d RMS^3) (App. "Lipschitzness of RMSNorm");
    with unit gain the tangent is that matrix applied to tx."""
    eps = 1e-3
    x, tx = rnd(1, d), rnd(2, d)
    rms = math.sqrt(float(np.mean(x * x)) + eps)
    J = np.eye(d) / rms - np.outer(x, x) / (d * rms ** 3)
    y, ty = orc.rmsnorm_jvp_fwd(x[None], tx[None], np.ones(d), eps)
    assert np.allclose(y[0], x / rms, rtol=1e-14, atol=1e-14)
    assert np.allclose(ty[0], J @ tx, rtol=1e-12, atol=1e-13)


def test_printed_jacobian_bound():
    """Every entry of that Jacobian is bounded by sqrt(2 / eps) in magnitude (same appendix)."""
    eps = 1e-2
    for seed, scale in ((3, 1e-3), (4, 1.0), (5, 1e3)):
        x = rnd(seed, 16, scale=scale)
        d = x.size
        for j in range(d):
            e = np.zeros(d)
            e[j] = 1.0
            _, col = orc.rmsnorm_jvp_fwd(x[None], e[None], np.ones(d), eps)
            assert np.all(np.abs(col) <= math.sqrt(2.0 / eps))


# ---------------------------------------------------------------------------- 2. finite differences
def plain_rmsnorm(x, g, eps):
    return g * x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)


@pytest.mark.parametrize("rows,d", [(1, 1), (3, 5), (4, 72)])
def test_tangent_is_directional_derivative(rows, d):
    x, tx, g, _, _ = case(10, rows, d)
    eps, h = 1e-4, 1e-5
    fd = (plain_rmsnorm(x + h * tx, g, eps) - plain_rmsnorm(x - h * tx, g, eps)) / (2 * h)
    y, ty = orc.rmsnorm_jvp_fwd(x, tx, g, eps)
    assert np.allclose(y, plain_rmsnorm(x, g, eps), rtol=1e-14, atol=1e-14)
    assert np.allclose(ty, fd, rtol=1e-7, atol=1e-8)


def loss(x, tx, g, eps, gy, gty, h=1e-5):
    """<gy, y> + <gty, ty> with ty itself by central differences of the plain definition."""
    y = plain_rmsnorm(x, g, eps)
    ty = (plain_rmsnorm(x + h * tx, g, eps) - plain_rmsnorm(x - h * tx, g, eps)) / (2 * h)
    return float(np.sum(gy * y) + np.sum(gty * ty))


@pytest.mark.parametrize("rows,d", [(1, 2), (2, 5), (3, 16)])
def test_every_gradient_entry_by_finite_differences(rows, d):
    x, tx, g, gy, gty = case(20, rows, d)
    eps, h = 1e-3, 1e-4
    gx, gtx, gg = orc.rmsnorm_jvp_bwd(x, tx, g, eps, gy, gty)
    for name, arr, grad in (("x", x, gx), ("tx", tx, gtx), ("g", g, gg)):
        for idx in np.ndindex(arr.shape):
            p = [a.copy() for a in (x, tx, g)]
            k = ("x", "tx", "g").index(name)
            p[k][idx] += h
            up = loss(p[0], p[1], p[2], eps, gy, gty)
            p[k][idx] -= 2 * h
            dn = loss(p[0], p[1], p[2], eps, gy, gty)
            fd = (up - dn) / (2 * h)
            assert abs(fd - grad[idx]) <= 2e-5 * max(1.0, abs(grad[idx])), (name, idx, fd, grad[idx])


# ---------------------------------------------------------------------------- 3. an independent mechanism
def test_against_torch_rms_norm_jvp_and_autograd():
    rows, d, eps = 6, 24, 1e-5
    x, tx, g, gy, gty = case(30, rows, d)
    T = lambda a: torch.tensor(a, dtype=torch.float64)
    xt, txt, gt = T(x).requires_grad_(True), T(tx).requires_grad_(True), T(g).requires_grad_(True)
    f = lambda xx: torch.nn.functional.rms_norm(xx, (d,), weight=gt, eps=eps)
    y, ty = torch.func.jvp(f, (xt,), (txt,))
    oy, oty = orc.rmsnorm_jvp_fwd(x, tx, g, eps)
    assert np.allclose(oy, y.detach().numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(oty, ty.detach().numpy(), rtol=1e-11, atol=1e-12)
    (y * T(gy)).sum().add((ty * T(gty)).sum()).backward()
    gx, gtx, gg = orc.rmsnorm_jvp_bwd(x, tx, g, eps, gy, gty)
    assert np.allclose(gx, xt.grad.numpy(), rtol=1e-10, atol=1e-11)
    assert np.allclose(gtx, txt.grad.numpy(), rtol=1e-10, atol=1e-11)
    assert np.allclose(gg, gt.grad.numpy(), rtol=1e-10, atol=1e-11)


# ---------------------------------------------------------------------------- 4. closed form by hand
def test_two_element_closed_form():
    """x = (3, 4), eps = 0: RMS = 5 / sqrt 2, y = (3, 4) sqrt 2 / 5.  Along tx = (1, 0): mean(x tx) = 3/2 and
    ty = tx / RMS - x (3/2) / RMS^3 = (16, -12) sqrt 2 / 125 (orthogonal to x, as scale invariance demands).
    With gain (2, 1/2) both double and halve.  For gy = (1, 0), gty = 0: the gradient of y_1 = g_1 x_1 / RMS is
    g_1 (1 / RMS - x_1^2 / (2 RMS^3), - x_1 x_2 / (2 RMS^3)) = 2 sqrt 2 (16, -12) / 125."""
    r2 = math.sqrt(2.0)
    x, tx, g = np.array([[3.0, 4.0]]), np.array([[1.0, 0.0]]), np.array([2.0, 0.5])
    y, ty = orc.rmsnorm_jvp_fwd(x, tx, g, 0.0)
    assert np.allclose(y[0], [2 * 3 * r2 / 5, 0.5 * 4 * r2 / 5], rtol=1e-15)
    assert np.allclose(ty[0], [2 * 16 * r2 / 125, -0.5 * 12 * r2 / 125], rtol=1e-14)
    gx, gtx, gg = orc.rmsnorm_jvp_bwd(x, tx, g, 0.0, np.array([[1.0, 0.0]]), np.zeros((1, 2)))
    assert np.allclose(gx[0], [2 * r2 * 16 / 125, -2 * r2 * 12 / 125], rtol=1e-14)
    assert np.allclose(gtx[0], [0.0, 0.0], atol=1e-16)
    assert np.allclose(gg, [3 * r2 / 5, 0.0], rtol=1e-15)


# ---------------------------------------------------------------------------- 5. invariants
def test_unit_rms_and_scale_invariance_without_eps():
    x, tx, g, gy, gty = case(40, 5, 12)
    y, ty = orc.rmsnorm_jvp_fwd(x, tx, g, 0.0)
    assert np.allclose(np.mean((y / g) ** 2, axis=-1), 1.0, rtol=1e-14)
    y2, _ = orc.rmsnorm_jvp_fwd(3.7 * x, tx, g, 0.0)
    assert np.allclose(y, y2, rtol=1e-14)
    _, t_along_x = orc.rmsnorm_jvp_fwd(x, x, g, 0.0)   # moving along x does not change x / RMS(x)
    assert np.allclose(t_along_x, 0.0, atol=1e-14)
    # y(c x), ty(c x, c tx) do not depend on c, so the derivative of the loss along (x, tx) vanishes
    gx, gtx, _ = orc.rmsnorm_jvp_bwd(x, tx, g, 0.0, gy, gty)
    assert np.allclose(np.sum(gx * x + gtx * tx, axis=-1), 0.0, atol=1e-12)


def test_tangent_is_linear_and_zero_for_zero():
    x, tx, g, _, _ = case(50, 4, 9)
    tx2 = rnd(55, 4, 9)
    _, a = orc.rmsnorm_jvp_fwd(x, tx, g, 1e-3)
    _, b = orc.rmsnorm_jvp_fwd(x, tx2, g, 1e-3)
    _, ab = orc.rmsnorm_jvp_fwd(x, 2.0 * tx - 3.0 * tx2, g, 1e-3)
    assert np.allclose(ab, 2.0 * a - 3.0 * b, rtol=1e-12, atol=1e-13)
    _, z = orc.rmsnorm_jvp_fwd(x, np.zeros_like(x), g, 1e-3)
    assert np.all(z == 0.0)


def test_rows_are_independent_and_gain_gradient_sums_over_rows():
    x, tx, g, gy, gty = case(60, 6, 8)
    gx, gtx, gg = orc.rmsnorm_jvp_bwd(x, tx, g, 1e-4, gy, gty)
    acc = np.zeros_like(g)
    for r in range(6):
        a, b, c = orc.rmsnorm_jvp_bwd(x[r:r + 1], tx[r:r + 1], g, 1e-4, gy[r:r + 1], gty[r:r + 1])
        assert np.allclose(a[0], gx[r], rtol=1e-13, atol=1e-14) and np.allclose(b[0], gtx[r], rtol=1e-13, atol=1e-14)
        acc += c
    assert np.allclose(acc, gg, rtol=1e-13, atol=1e-14)
    # batched shapes: leading axes are all rows
    y4, ty4 = orc.rmsnorm_jvp_fwd(x.reshape(1, 2, 3, 8), tx.reshape(1, 2, 3, 8), g, 1e-4)
    y2, ty2 = orc.rmsnorm_jvp_fwd(x, tx, g, 1e-4)
    assert np.array_equal(y4.reshape(6, 8), y2) and np.array_equal(ty4.reshape(6, 8), ty2)
