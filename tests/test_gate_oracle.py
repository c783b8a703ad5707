"""Pins of the normalised residual-gate oracle to things other than itself: finite differences of the plain
definition, torch's own rms_norm under forward- and reverse-mode autodiff, and special cases.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import gate_oracle as orc


def rnd(seed, *shape, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def case(seed, B, T, C):
    return (rnd(seed, B, T, C), rnd(seed + 1, B, T, C, scale=0.6), rnd(seed + 2, B, T, C), rnd(seed + 3, B, T, C, scale=0.7),
            rnd(seed + 4, B, C), rnd(seed + 5, B, C, scale=0.5), rnd(seed + 6, B, T, C), rnd(seed + 7, B, T, C))


def plain(x, h, c, eps):
    """x + RMSNorm^-(c) o h, written out (App. "Full Description of Normalization of Modulation")."""
    n = lambda v: v / np.sqrt(np.mean(v * v, axis=-1, keepdims=True) + eps)
    return x + n(c)[:, None, :] * h


@pytest.mark.parametrize("B,T,C", [(1, 1, 2), (2, 3, 5), (2, 4, 24)])
def test_tangent_is_directional_derivative(B, T, C):
    x, tx, h, th, c, tc, _, _ = case(10, B, T, C)
    eps, d = 1e-4, 1e-5
    fd = (plain(x + d * tx, h + d * th, c + d * tc, eps) - plain(x - d * tx, h - d * th, c - d * tc, eps)) / (2 * d)
    z, tz = orc.gate_jvp_fwd(x, tx, h, th, c, tc, eps)
    assert np.allclose(z, plain(x, h, c, eps), rtol=1e-13, atol=1e-13)
    assert np.allclose(tz, fd, rtol=1e-7, atol=1e-8)


def loss(p, eps, gz, gtz, d=1e-5):
    x, tx, h, th, c, tc = p
    z = plain(x, h, c, eps)
    tz = (plain(x + d * tx, h + d * th, c + d * tc, eps) - plain(x - d * tx, h - d * th, c - d * tc, eps)) / (2 * d)
    return float(np.sum(gz * z) + np.sum(gtz * tz))


@pytest.mark.parametrize("B,T,C", [(1, 1, 2), (2, 3, 4), (1, 5, 6)])
def test_every_gradient_entry_by_finite_differences(B, T, C):
    x, tx, h, th, c, tc, gz, gtz = case(20, B, T, C)
    eps, d = 1e-3, 1e-4
    grads = orc.gate_jvp_bwd(x, tx, h, th, c, tc, eps, gz, gtz)
    params = [x, tx, h, th, c, tc]
    for k, (arr, grad) in enumerate(zip(params, grads)):
        for idx in np.ndindex(arr.shape):
            p = [v.copy() for v in params]
            p[k][idx] += d
            up = loss(p, eps, gz, gtz)
            p[k][idx] -= 2 * d
            dn = loss(p, eps, gz, gtz)
            fd = (up - dn) / (2 * d)
            assert abs(fd - grad[idx]) <= 3e-5 * max(1.0, abs(grad[idx])), (k, idx, fd, grad[idx])


def test_against_torch_rms_norm_jvp_and_autograd():
    B, T, C, eps = 2, 5, 16, 1e-5
    vals = case(30, B, T, C)
    T64 = lambda v: torch.tensor(v, dtype=torch.float64)
    x, tx, h, th, c, tc = (T64(v).requires_grad_(True) for v in vals[:6])
    f = lambda xx, hh, cc: xx + torch.nn.functional.rms_norm(cc, (C,), eps=eps)[:, None, :] * hh
    z, tz = torch.func.jvp(f, (x, h, c), (tx, th, tc))
    oz, otz = orc.gate_jvp_fwd(*vals[:6], eps)
    assert np.allclose(oz, z.detach().numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(otz, tz.detach().numpy(), rtol=1e-11, atol=1e-12)
    ((z * T64(vals[6])).sum() + (tz * T64(vals[7])).sum()).backward()
    got = orc.gate_jvp_bwd(*vals[:6], eps, vals[6], vals[7])
    for g, t in zip(got, (x, tx, h, th, c, tc)):
        assert np.allclose(g, t.grad.numpy(), rtol=1e-10, atol=1e-11)


def test_constant_gate_zero_tangents_and_linearity():
    B, T, C = 2, 3, 8
    x, tx, h, th, c, tc, gz, gtz = case(40, B, T, C)
    # a constant vector normalises to ones (eps = 0): the gate is then open, z = x + h; minus ones: z = x - h
    z, _ = orc.gate_jvp_fwd(x, tx, h, th, np.full((B, C), 3.0), tc, 0.0)
    assert np.allclose(z, x + h, rtol=1e-13)
    z, _ = orc.gate_jvp_fwd(x, tx, h, th, np.full((B, C), -0.5), tc, 0.0)
    assert np.allclose(z, x - h, rtol=1e-13)
    _, t0 = orc.gate_jvp_fwd(x, np.zeros_like(x), h, np.zeros_like(h), c, np.zeros_like(c), 1e-3)
    assert np.all(t0 == 0.0)
    # the gate is scale invariant at eps = 0, so a tangent of c along c changes nothing: tz = tx + ch th
    _, t1 = orc.gate_jvp_fwd(x, tx, h, th, c, 0.3 * c, 0.0)
    n = c / np.sqrt(np.mean(c * c, axis=-1, keepdims=True))
    assert np.allclose(t1, tx + n[:, None, :] * th, rtol=1e-12, atol=1e-13)
    # tangents enter linearly
    _, ta = orc.gate_jvp_fwd(x, tx, h, th, c, tc, 1e-3)
    _, tb = orc.gate_jvp_fwd(x, 2 * tx, h, 2 * th, c, 2 * tc, 1e-3)
    assert np.allclose(tb, 2 * ta, rtol=1e-12, atol=1e-13)


def test_stream_gradients_pass_through_and_gate_gradients_sum_over_tokens():
    B, T, C = 2, 4, 6
    x, tx, h, th, c, tc, gz, gtz = case(50, B, T, C)
    full = orc.gate_jvp_bwd(x, tx, h, th, c, tc, 1e-4, gz, gtz)
    assert np.array_equal(full[0], gz) and np.array_equal(full[1], gtz)
    for bb in range(B):
        acc = [np.zeros(C) for _ in range(2)]
        for t in range(T):
            s = (slice(bb, bb + 1), slice(t, t + 1))
            one = orc.gate_jvp_bwd(x[s], tx[s], h[s], th[s], c[bb:bb + 1], tc[bb:bb + 1], 1e-4, gz[s], gtz[s])
            for k in (2, 3):
                assert np.allclose(one[k][0, 0], full[k][bb, t], rtol=1e-12, atol=1e-13)
            for k in range(2):
                acc[k] += one[4 + k][0]
        for k in range(2):
            assert np.allclose(acc[k], full[4 + k][bb], rtol=1e-12, atol=1e-13)


def test_planted_mistakes_fail_a_pin():
    """A dropped term or a swapped operand in the tangent or in the gate's gradient shows against finite differences."""
    B, T, C = 1, 3, 4
    x, tx, h, th, c, tc, gz, gtz = case(60, B, T, C)
    eps, d = 1e-3, 1e-5
    fd = (plain(x + d * tx, h + d * th, c + d * tc, eps) - plain(x - d * tx, h - d * th, c - d * tc, eps)) / (2 * d)
    from oracle import rmsnorm_oracle as rn
    ch, tch = rn.rmsnorm_jvp_fwd(c, tc, np.ones(C), eps)
    wrong = [tx + ch[:, None, :] * th,                          # the gate's own tangent dropped
             tx + tch[:, None, :] * th + ch[:, None, :] * h,    # h and th swapped
             tch[:, None, :] * h + ch[:, None, :] * th]         # the stream's tangent dropped
    for w in wrong:
        assert not np.allclose(w, fd, rtol=1e-5, atol=1e-6)
