"""Pins of the linear-layer oracle to things other than itself: finite differences of the plain map, scalar loops,
torch's own linear under forward- and reverse-mode autodiff, hand-worked cases, planted mistakes.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import linear_oracle as orc


def rnd(seed, *shape, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def case(seed, R, K, F):
    return (rnd(seed, R, K), rnd(seed + 1, R, K, scale=0.6), rnd(seed + 2, F, K, scale=0.5), rnd(seed + 3, F),
            rnd(seed + 4, R, F), rnd(seed + 5, R, F, scale=0.8))


def plain(x, w, b):
    """y_rf = sum_k W_fk x_rk + b_f, in scalar loops."""
    R, K = x.shape
    F = w.shape[0]
    y = np.zeros((R, F))
    for r in range(R):
        for f in range(F):
            s = b[f]
            for k in range(K):
                s += w[f, k] * x[r, k]
            y[r, f] = s
    return y


@pytest.mark.parametrize("R,K,F", [(1, 1, 1), (3, 4, 2), (5, 7, 6)])
def test_forward_is_the_plain_map_and_the_tangent_its_directional_derivative(R, K, F):
    x, tx, w, b, _, _ = case(10, R, K, F)
    y, ty = orc.linear_jvp_fwd(x, tx, w, b)
    assert np.allclose(y, plain(x, w, b), rtol=1e-13, atol=1e-13)
    d = 1e-5
    fd = (plain(x + d * tx, w, b) - plain(x - d * tx, w, b)) / (2 * d)
    assert np.allclose(ty, fd, rtol=1e-8, atol=1e-9)
    # no bias: the same without b
    y0, ty0 = orc.linear_jvp_fwd(x, tx, w, None)
    assert np.allclose(y0, y - b[None, :], rtol=1e-13, atol=1e-13) and np.array_equal(ty0, ty)


def loss(p, gy, gty, d=1e-5):
    x, tx, w, b = p
    y = plain(x, w, b)
    ty = (plain(x + d * tx, w, b) - plain(x - d * tx, w, b)) / (2 * d)
    return float(np.sum(gy * y) + np.sum(gty * ty))


@pytest.mark.parametrize("R,K,F", [(1, 1, 1), (2, 3, 2), (4, 3, 5)])
def test_every_gradient_entry_by_finite_differences(R, K, F):
    x, tx, w, b, gy, gty = case(20, R, K, F)
    grads = orc.linear_jvp_bwd(x, tx, w, gy, gty)
    params = [x, tx, w, b]
    d = 1e-4
    for k, (arr, grad) in enumerate(zip(params, grads)):
        assert arr.shape == grad.shape
        for idx in np.ndindex(arr.shape):
            p = [v.copy() for v in params]
            p[k][idx] += d
            up = loss(p, gy, gty)
            p[k][idx] -= 2 * d
            dn = loss(p, gy, gty)
            fd = (up - dn) / (2 * d)
            assert abs(fd - grad[idx]) <= 2e-6 * max(1.0, abs(grad[idx])), (k, idx, fd, grad[idx])


def test_against_torch_linear_jvp_and_autograd():
    R, K, F = 6, 9, 5
    x, tx, w, b, gy, gty = case(30, R, K, F)
    T = lambda a: torch.tensor(a, dtype=torch.float64)
    wt, bt = T(w).requires_grad_(True), T(b).requires_grad_(True)
    xt, txt = T(x).requires_grad_(True), T(tx).requires_grad_(True)
    y, ty = torch.func.jvp(lambda v: torch.nn.functional.linear(v, wt, bt), (xt,), (txt,))
    oy, oty = orc.linear_jvp_fwd(x, tx, w, b)
    assert np.allclose(oy, y.detach().numpy(), rtol=1e-13, atol=1e-13)
    assert np.allclose(oty, ty.detach().numpy(), rtol=1e-13, atol=1e-13)
    L = (T(gy) * y).sum() + (T(gty) * ty).sum()
    g = torch.autograd.grad(L, (xt, txt, wt, bt))
    for mine, ref in zip(orc.linear_jvp_bwd(x, tx, w, gy, gty), g):
        assert np.allclose(mine, ref.numpy(), rtol=1e-12, atol=1e-12)


def test_hand_worked_case():
    """One token, two features in, one out: W = (2, -3), b = 5, x = (1, 4), tx = (0.5, -1): y = 2 - 12 + 5 = -5,
    ty = 1 + 3 = 4; with gy = 7, gty = -2: gx = 7 W, gtx = -2 W, gW = 7 x - 2 tx = (6, 30), gb = 7."""
    y, ty = orc.linear_jvp_fwd([[1.0, 4.0]], [[0.5, -1.0]], [[2.0, -3.0]], [5.0])
    assert y.tolist() == [[-5.0]] and ty.tolist() == [[4.0]]
    gx, gtx, gw, gb = orc.linear_jvp_bwd([[1.0, 4.0]], [[0.5, -1.0]], [[2.0, -3.0]], [[7.0]], [[-2.0]])
    assert gx.tolist() == [[14.0, -21.0]] and gtx.tolist() == [[-4.0, 6.0]]
    assert gw.tolist() == [[6.0, 30.0]] and gb.tolist() == [7.0]


def test_special_cases_and_invariants():
    R, K = 5, 6
    x, tx, _, b, gy, gty = case(40, R, K, K)
    eye = np.eye(K)
    y, ty = orc.linear_jvp_fwd(x, tx, eye, b)
    assert np.allclose(y, x + b[None, :]) and np.array_equal(ty, tx)          # identity weight
    w = rnd(41, 4, K)
    _, t0 = orc.linear_jvp_fwd(x, np.zeros_like(x), w, None)
    assert not t0.any()                                                        # zero tangent in, zero tangent out
    _, t1 = orc.linear_jvp_fwd(x, tx, w, None)
    _, t2 = orc.linear_jvp_fwd(x, -2.5 * tx, w, None)
    assert np.allclose(t2, -2.5 * t1, rtol=1e-13, atol=1e-13)                  # linear in the tangent
    _, t3 = orc.linear_jvp_fwd(x + 3.0, tx, w, b[:4])
    assert np.allclose(t3, t1, rtol=1e-13, atol=1e-13)                         # and independent of x and b
    # tokens are independent: the weight gradient is the sum of one-token gradients, gx of a token ignores the others
    gy4, gty4 = gy[:, :4], gty[:, :4]
    gx, gtx, gw, gb = orc.linear_jvp_bwd(x, tx, w, gy4, gty4)
    gw_sum, gb_sum = np.zeros_like(gw), np.zeros_like(gb)
    for r in range(R):
        a = orc.linear_jvp_bwd(x[r:r + 1], tx[r:r + 1], w, gy4[r:r + 1], gty4[r:r + 1])
        assert np.allclose(a[0][0], gx[r]) and np.allclose(a[1][0], gtx[r])
        gw_sum += a[2]
        gb_sum += a[3]
    assert np.allclose(gw_sum, gw, rtol=1e-12, atol=1e-12) and np.allclose(gb_sum, gb, rtol=1e-12, atol=1e-12)
    # the layer on the stacked rows [x; tx] is the forward and the tangent at once (what the kernels exploit)
    stacked, _ = orc.linear_jvp_fwd(np.concatenate([x, tx]), np.zeros((2 * R, K)), w, None)
    y5, ty5 = orc.linear_jvp_fwd(x, tx, w, None)
    assert np.allclose(stacked[:R], y5) and np.allclose(stacked[R:], ty5)


def _gradients_agree_with_finite_differences(bwd, fwd_has_bias_in_tangent=False):
    R, K, F = 3, 4, 3
    x, tx, w, b, gy, gty = case(50, R, K, F)
    grads = bwd(x, tx, w, gy, gty)
    params = [x, tx, w, b]
    d = 1e-4
    for k, (arr, grad) in enumerate(zip(params, grads)):
        for idx in np.ndindex(arr.shape):
            p = [v.copy() for v in params]
            p[k][idx] += d
            up = loss(p, gy, gty)
            p[k][idx] -= 2 * d
            dn = loss(p, gy, gty)
            if abs((up - dn) / (2 * d) - grad[idx]) > 2e-6 * max(1.0, abs(grad[idx])):
                return False
    return True


def test_planted_mistakes_are_caught():
    """Plausible slips planted in copies of the oracle's backward each fail the finite-difference pin, which the
    oracle itself passes; slips in the forward fail the scalar-loop and directional-derivative pins."""
    assert _gradients_agree_with_finite_differences(orc.linear_jvp_bwd)
    mutants = {
        "tangent term of gW dropped": lambda x, tx, w, gy, gty: (gy @ w, gty @ w, gy.T @ x, gy.sum(0)),
        "gW pairs gy with tx": lambda x, tx, w, gy, gty: (gy @ w, gty @ w, gy.T @ tx + gty.T @ x, gy.sum(0)),
        "gx and gtx swapped": lambda x, tx, w, gy, gty: (gty @ w, gy @ w, gy.T @ x + gty.T @ tx, gy.sum(0)),
        "bias gradient collects gty too": lambda x, tx, w, gy, gty: (gy @ w, gty @ w, gy.T @ x + gty.T @ tx, (gy + gty).sum(0)),
        "wrong sign on the tangent path": lambda x, tx, w, gy, gty: (gy @ w, -(gty @ w), gy.T @ x - gty.T @ tx, gy.sum(0)),
    }
    for name, m in mutants.items():
        assert not _gradients_agree_with_finite_differences(m), name
    # forward slips: a bias in the tangent, a transposed weight
    x, tx, w, b, _, _ = case(51, 3, 4, 4)
    y, ty = orc.linear_jvp_fwd(x, tx, w, b)
    d = 1e-5
    fd = (plain(x + d * tx, w, b) - plain(x - d * tx, w, b)) / (2 * d)
    assert np.allclose(ty, fd, rtol=1e-8, atol=1e-9) and not np.allclose(tx @ w.T + b[None, :], fd, rtol=1e-8, atol=1e-9)
    assert np.allclose(y, plain(x, w, b)) and not np.allclose(x @ w + b[None, :], plain(x, w, b))
