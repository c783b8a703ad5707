"""Pins of the activation oracle (tanh-form GELU with tangent and backward) to things other than itself.  CPU only."""
import numpy as np
import torch

from oracle import gelu_oracle as orc


def rnd(seed, *shape, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def test_against_torch_gelu_jvp_and_autograd():
    u, tu, ga, gta = rnd(1, 4000, scale=2.0), rnd(2, 4000), rnd(3, 4000), rnd(4, 4000)
    T64 = lambda v: torch.tensor(v, dtype=torch.float64)
    U, TU = T64(u).requires_grad_(True), T64(tu).requires_grad_(True)
    f = lambda x: torch.nn.functional.gelu(x, approximate="tanh")
    a, ta = torch.func.jvp(f, (U,), (TU,))
    oa, ota = orc.gelu_jvp_fwd(u, tu)
    assert np.allclose(oa, a.detach().numpy(), rtol=1e-12, atol=1e-14)
    assert np.allclose(ota, ta.detach().numpy(), rtol=1e-12, atol=1e-14)
    ((a * T64(ga)).sum() + (ta * T64(gta)).sum()).backward()
    gu, gtu = orc.gelu_jvp_bwd(u, tu, ga, gta)
    assert np.allclose(gu, U.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(gtu, TU.grad.numpy(), rtol=1e-12, atol=1e-14)


def plain(u):
    """The formula as DiT's MLP uses it, written out."""
    return 0.5 * u * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (u + 0.044715 * u ** 3)))


def test_finite_differences():
    u, tu, ga, gta = rnd(5, 300, scale=1.5), rnd(6, 300), rnd(7, 300), rnd(8, 300)
    h = 1e-5
    a, ta = orc.gelu_jvp_fwd(u, tu)
    assert np.allclose(a, plain(u), rtol=1e-14, atol=1e-15)
    assert np.allclose(ta, (plain(u + h * tu) - plain(u - h * tu)) / (2 * h), rtol=1e-7, atol=1e-9)
    # the loss is a sum over independent elements: perturb all at once, per input
    d = 1e-4
    tang = lambda uu, tt: (plain(uu + h * tt) - plain(uu - h * tt)) / (2 * h)
    L = lambda uu, tt: ga * plain(uu) + gta * tang(uu, tt)     # per element
    gu, gtu = orc.gelu_jvp_bwd(u, tu, ga, gta)
    assert np.allclose(gu, (L(u + d, tu) - L(u - d, tu)) / (2 * d), rtol=2e-5, atol=2e-6)
    assert np.allclose(gtu, (L(u, tu + d) - L(u, tu - d)) / (2 * d), rtol=2e-5, atol=2e-6)


def test_values_limits_and_identities():
    a, ta = orc.gelu_jvp_fwd(np.zeros(3), np.array([1.0, -2.0, 0.5]))
    assert np.all(a == 0.0) and np.allclose(ta, [0.5, -1.0, 0.25], rtol=1e-15)      # gelu(0) = 0, gelu'(0) = 1/2
    big = np.array([12.0, 30.0])
    a, ta = orc.gelu_jvp_fwd(big, np.ones(2))
    assert np.allclose(a, big, rtol=1e-14) and np.allclose(ta, 1.0, rtol=1e-12)     # identity far to the right
    a, ta = orc.gelu_jvp_fwd(-big, np.ones(2))
    assert np.allclose(a, 0.0, atol=1e-14) and np.allclose(ta, 0.0, atol=1e-12)     # zero far to the left
    u, tu = rnd(9, 200, scale=2.0), rnd(10, 200)
    ap, tap = orc.gelu_jvp_fwd(u, tu)
    am, tam = orc.gelu_jvp_fwd(-u, tu)
    assert np.allclose(ap - am, u, rtol=1e-13, atol=1e-14)                          # tanh is odd: gelu(u) - gelu(-u) = u
    assert np.allclose(tap + tam, tu, rtol=1e-13, atol=1e-14)                       # hence gelu'(u) + gelu'(-u) = 1
    _, t2 = orc.gelu_jvp_fwd(u, 3.0 * tu)
    assert np.allclose(t2, 3.0 * tap, rtol=1e-14)
    # gelu'' at 0 is 2 k (from the series u/2 + k u^2 / 2 + ...): the gradient of u through the tangent output
    gu, gtu = orc.gelu_jvp_bwd(np.zeros(1), np.ones(1), np.zeros(1), np.ones(1))
    assert np.allclose(gu, 2.0 * np.sqrt(2.0 / np.pi) * 0.5, rtol=1e-14) and np.allclose(gtu, 0.5)


def test_planted_mistakes_fail_a_pin():
    u, tu = rnd(11, 100, scale=1.5), rnd(12, 100)
    h = 1e-5
    fd = (plain(u + h * tu) - plain(u - h * tu)) / (2 * h)
    k, c = np.sqrt(2.0 / np.pi), 0.044715
    t = np.tanh(k * (u + c * u ** 3))
    wrong = [0.5 * tu * (1 + t),                                              # the tanh's own derivative dropped
             0.5 * tu * (1 + t) + 0.5 * u * (1 - t * t) * k * tu,             # the cubic term's derivative dropped
             0.5 * tu * (1 + t) + 0.5 * u * (1 - t) * k * (1 + 3 * c * u ** 2) * tu]   # 1 - t instead of 1 - t^2
    for w in wrong:
        assert not np.allclose(w, fd, rtol=1e-4, atol=1e-5)
