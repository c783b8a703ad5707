"""Pins of the block oracle (the chain of the per-operation oracles) to things other than itself: the same block
written with torch's own operators under torch.func.jvp and autograd in float64, finite differences of the forward
for the tangent, and planted wiring mistakes.  CPU only."""
import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

from oracle import block_oracle as orc

EPS, QK_EPS = 1e-5, 1e-6


def make(seed, B, T, H, d, hidden):
    rng = np.random.default_rng(seed)
    C = H * d
    n = lambda *s, scale=1.0: rng.standard_normal(s) * scale
    x, tx = n(B, T, C), n(B, T, C, scale=0.7)
    mods = {k: n(B, C) for k in orc.MODS}
    tmods = {k: n(B, C, scale=0.5) for k in orc.MODS}
    params = {"wqkv": n(3 * C, C, scale=C ** -0.5), "bqkv": n(3 * C, scale=0.1), "gq": 1 + 0.2 * n(d), "gk": 1 + 0.2 * n(d),
              "wo": n(C, C, scale=C ** -0.5), "bo": n(C, scale=0.1), "w1": n(hidden, C, scale=C ** -0.5),
              "b1": n(hidden, scale=0.1), "w2": n(C, hidden, scale=hidden ** -0.5), "b2": n(C, scale=0.1)}
    return x, tx, mods, tmods, params, n(B, T, C), n(B, T, C)


def torch_block(x, mods, p, H):
    """The block of App. "Full Description of Normalization of Modulation" with torch's operators."""
    B, T, C = x.shape
    d = C // H
    nrm = lambda v: Fn.rms_norm(v, (v.shape[-1],), eps=EPS)
    u1 = nrm(x) * nrm(mods["a1"])[:, None, :] + nrm(mods["b1"])[:, None, :]
    qkv = Fn.linear(u1, p["wqkv"], p["bqkv"]).reshape(B, T, 3, H, d).permute(2, 0, 3, 1, 4)
    q = Fn.rms_norm(qkv[0], (d,), weight=p["gq"], eps=QK_EPS)
    k = Fn.rms_norm(qkv[1], (d,), weight=p["gk"], eps=QK_EPS)
    # (softmax attention in torch's plain operators: its fused CPU kernel has no forward-mode derivative)
    o = (torch.softmax(q @ k.transpose(-1, -2) * d ** -0.5, dim=-1) @ qkv[2]).transpose(1, 2).reshape(B, T, C)
    x1 = x + nrm(mods["c1"])[:, None, :] * Fn.linear(o, p["wo"], p["bo"])
    u2 = nrm(x1) * nrm(mods["a2"])[:, None, :] + nrm(mods["b2"])[:, None, :]
    h2 = Fn.linear(Fn.gelu(Fn.linear(u2, p["w1"], p["b1"]), approximate="tanh"), p["w2"], p["b2"])
    return x1 + nrm(mods["c2"])[:, None, :] * h2


@pytest.mark.parametrize("B,T,H,d,hidden", [(1, 3, 1, 4, 8), (2, 5, 2, 4, 24)])
def test_against_torch_operators_under_jvp_and_autograd(B, T, H, d, hidden):
    x, tx, mods, tmods, params, gz, gtz = make(1, B, T, H, d, hidden)
    T64 = lambda a: torch.tensor(a, dtype=torch.float64)
    xt, txt = T64(x).requires_grad_(True), T64(tx).requires_grad_(True)
    mt = {k: T64(v).requires_grad_(True) for k, v in mods.items()}
    tmt = {k: T64(v).requires_grad_(True) for k, v in tmods.items()}
    pt = {k: T64(v).requires_grad_(True) for k, v in params.items()}
    names = list(orc.MODS)
    fn = lambda xv, *mv: torch_block(xv, dict(zip(names, mv)), pt, H)
    z, tz = torch.func.jvp(fn, (xt, *[mt[k] for k in names]), (txt, *[tmt[k] for k in names]))
    oz, otz = orc.block_jvp_fwd(x, tx, mods, tmods, params, H, EPS, QK_EPS)
    assert np.allclose(oz, z.detach().numpy(), rtol=1e-10, atol=1e-11)
    assert np.allclose(otz, tz.detach().numpy(), rtol=1e-10, atol=1e-11)
    L = (T64(gz) * z).sum() + (T64(gtz) * tz).sum()
    wrt = [xt, txt] + [mt[k] for k in names] + [tmt[k] for k in names] + [pt[k] for k in orc.PARAMS]
    grads = torch.autograd.grad(L, wrt)
    g = orc.block_jvp_bwd(x, tx, mods, tmods, params, H, EPS, QK_EPS, gz, gtz)
    key = {"b1": "mb1", "b2": "mb2"}   # the modulation shifts, as the oracle names them beside the MLP's biases
    mine = [g["x"], g["tx"]] + [g[key.get(k, k)] for k in names] + [g["t" + key.get(k, k)] for k in names] + \
           [g[k] for k in orc.PARAMS]
    for i, (a, b) in enumerate(zip(mine, grads)):
        assert a.shape == tuple(b.shape)
        assert np.allclose(a, b.numpy(), rtol=1e-9, atol=1e-10), i


def test_tangent_is_the_directional_derivative_of_the_forward():
    x, tx, mods, tmods, params, _, _ = make(2, 2, 4, 2, 4, 16)
    zero = {k: np.zeros_like(v) for k, v in mods.items()}
    fwd = lambda e: orc.block_jvp_fwd(x + e * tx, np.zeros_like(x), {k: mods[k] + e * tmods[k] for k in mods}, zero, params,
                                      2, EPS, QK_EPS)[0]
    e = 1e-5
    fd = (fwd(e) - fwd(-e)) / (2 * e)
    _, tz = orc.block_jvp_fwd(x, tx, mods, tmods, params, 2, EPS, QK_EPS)
    assert np.allclose(tz, fd, rtol=1e-6, atol=1e-8)
    # zero tangents in, zero tangent out
    _, t0 = orc.block_jvp_fwd(x, np.zeros_like(x), mods, zero, params, 2, EPS, QK_EPS)
    assert not t0.any()


def test_planted_wiring_mistakes_are_caught(monkeypatch):
    """Slips in the chain (heads split in the wrong order, a residual gradient dropped, the second gate fed the
    first stream) change outputs or gradients that the torch pin fixes."""
    x, tx, mods, tmods, params, gz, gtz = make(3, 1, 4, 2, 4, 8)
    z, tz = orc.block_jvp_fwd(x, tx, mods, tmods, params, 2, EPS, QK_EPS)
    g = orc.block_jvp_bwd(x, tx, mods, tmods, params, 2, EPS, QK_EPS, gz, gtz)
    # 1. features split as [H, 3, d] instead of [3, H, d]
    def bad_split(y, H):
        B, T, C3 = y.shape
        d = C3 // (3 * H)
        y5 = y.reshape(B, T, H, 3, d)
        return tuple(np.ascontiguousarray(y5[:, :, :, i].transpose(0, 2, 1, 3)) for i in range(3))
    with monkeypatch.context() as mp:
        mp.setattr(orc, "_split_heads", bad_split)
        z2, _ = orc.block_jvp_fwd(x, tx, mods, tmods, params, 2, EPS, QK_EPS)
    assert not np.allclose(z2, z)
    # 2. the adaln's gradient of the stream not added to the residual connection's
    from oracle import adaln_oracle
    real = adaln_oracle.adaln_jvp_bwd
    def dropped(*a):
        r = list(real(*a))
        r[0], r[1] = np.zeros_like(r[0]), np.zeros_like(r[1])
        return tuple(r)
    with monkeypatch.context() as mp:
        mp.setattr(adaln_oracle, "adaln_jvp_bwd", dropped)
        g2 = orc.block_jvp_bwd(x, tx, mods, tmods, params, 2, EPS, QK_EPS, gz, gtz)
    assert not np.allclose(g2["x"], g["x"]) and not np.allclose(g2["wqkv"], g["wqkv"])
