"""Pins for the float64 oracle: everything here checks oracle/ against something
that is not the oracle -- finite differences of the definition, scalar loops,
closed forms, PyTorch's own CPU attention / JVP / autograd, the paper's
Step 1-6 closed forms, invariants and special cases.  CPU only.
"""
import math

import numpy as np
import pytest
import torch

from oracle import tvmattn_oracle as orc


def rnd(seed, *shape, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def head_inputs(seed, M, N, d):
    r = np.random.default_rng(seed)
    Q, Qd = r.standard_normal((M, d)), r.standard_normal((M, d))
    K, V, Kd, Vd = (r.standard_normal((N, d)) for _ in range(4))
    G, Gd = r.standard_normal((M, d)), r.standard_normal((M, d))
    return Q, K, V, Qd, Kd, Vd, G, Gd


def plain_attention(Q, K, V, a):
    """Eq. (sdpa) written out once more, only as the function to difference."""
    z = a * Q @ K.T
    z = z - z.max(axis=1, keepdims=True)
    e = np.exp(z)
    return (e / e.sum(axis=1, keepdims=True)) @ V


# ----------------------------------------------------------------------------
# 1. central finite differences of the definition
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("M,N,d", [(3, 5, 4), (6, 6, 2), (1, 7, 3), (5, 1, 3)])
def test_tangent_is_directional_derivative(M, N, d):
    Q, K, V, Qd, Kd, Vd, _, _ = head_inputs(1, M, N, d)
    a = 1.0 / math.sqrt(d)
    O, Od, _, _ = orc.attn_jvp_fwd_head(Q, K, V, Qd, Kd, Vd)
    eps = 1e-5
    fd = (plain_attention(Q + eps * Qd, K + eps * Kd, V + eps * Vd, a)
          - plain_attention(Q - eps * Qd, K - eps * Kd, V - eps * Vd, a)) / (2 * eps)
    assert np.allclose(O, plain_attention(Q, K, V, a), rtol=0, atol=1e-14)
    assert np.abs(Od - fd).max() <= 1e-8 * max(1.0, np.abs(fd).max())


def fd_tangent(Q, K, V, Qd, Kd, Vd, a, eps=1e-4):
    """Five-point central difference of eq. (sdpa) along the tangent direction (error O(eps^4))."""
    f = lambda t: plain_attention(Q + t * Qd, K + t * Kd, V + t * Vd, a)
    return (-f(2 * eps) + 8 * f(eps) - 8 * f(-eps) + f(-2 * eps)) / (12 * eps)


def loss_fd(Q, K, V, Qd, Kd, Vd, G, Gd, a):
    """L = <G, attn> + <Gd, d/deps attn>, built from eq. (sdpa) alone (no oracle call)."""
    return float((G * plain_attention(Q, K, V, a)).sum()
                 + (Gd * fd_tangent(Q, K, V, Qd, Kd, Vd, a)).sum())


@pytest.mark.parametrize("M,N,d", [(3, 4, 2), (4, 3, 3)])
def test_every_gradient_entry_by_finite_differences(M, N, d):
    """Every entry of all six gradients against a central difference of L, where L
    itself is assembled only from eq. (sdpa) (the tangent by a 5-point stencil)."""
    args = list(head_inputs(2, M, N, d))
    a = 1.0 / math.sqrt(d)
    grads = orc.attn_jvp_bwd_head(*args)
    order = [0, 1, 2, 3, 4, 5]           # dQ,dK,dV,dQd,dKd,dVd <-> Q,K,V,Qd,Kd,Vd
    h = 1e-3
    for gi, ai in enumerate(order):
        X = args[ai]
        for idx in np.ndindex(*X.shape):
            old = X[idx]
            vals = []
            for t in (2 * h, h, -h, -2 * h):
                X[idx] = old + t
                vals.append(loss_fd(*args, a))
            X[idx] = old
            fd = (-vals[0] + 8 * vals[1] - 8 * vals[2] + vals[3]) / (12 * h)
            assert abs(grads[gi][idx] - fd) <= 2e-6 * max(1.0, abs(fd)), (gi, idx, grads[gi][idx], fd)


def test_gradients_random_directions_larger():
    """Directional derivative of L (oracle forward) along random directions, N=24,d=8."""
    args = list(head_inputs(3, 24, 24, 8))
    grads = orc.attn_jvp_bwd_head(*args)

    def L(xs):
        O, Od, _, _ = orc.attn_jvp_fwd_head(*xs[:6])
        return float((xs[6] * O).sum() + (xs[7] * Od).sum())

    r = np.random.default_rng(7)
    for _ in range(4):
        dirs = [r.standard_normal(x.shape) for x in args[:6]]
        eps = 1e-5
        plus = [x + eps * u for x, u in zip(args[:6], dirs)] + args[6:]
        minus = [x - eps * u for x, u in zip(args[:6], dirs)] + args[6:]
        fd = (L(plus) - L(minus)) / (2 * eps)
        an = sum(float((g * u).sum()) for g, u in zip(grads, dirs))
        assert abs(fd - an) <= 1e-7 * max(1.0, abs(an))


# ----------------------------------------------------------------------------
# 2. scalar loops on tiny inputs (no numpy linear algebra at all)
# ----------------------------------------------------------------------------
def scalar_forward(Q, K, V, Qd, Kd, Vd):
    M, d = len(Q), len(Q[0])
    N = len(K)
    a = 1.0 / math.sqrt(d)
    O = [[0.0] * d for _ in range(M)]
    Od = [[0.0] * d for _ in range(M)]
    for i in range(M):
        z = [a * sum(Q[i][r] * K[j][r] for r in range(d)) for j in range(N)]
        zd = [a * sum(Qd[i][r] * K[j][r] + Q[i][r] * Kd[j][r] for r in range(d)) for j in range(N)]
        den = sum(math.exp(x) for x in z)
        p = [math.exp(x) / den for x in z]
        mb = sum(p[j] * zd[j] for j in range(N))
        for c in range(d):
            O[i][c] = sum(p[j] * V[j][c] for j in range(N))
            Od[i][c] = sum(p[j] * (zd[j] - mb) * V[j][c] + p[j] * Vd[j][c] for j in range(N))
    return O, Od


@pytest.mark.parametrize("M,N,d", [(2, 3, 2), (4, 4, 1), (1, 2, 2)])
def test_forward_against_scalar_loops(M, N, d):
    Q, K, V, Qd, Kd, Vd, _, _ = head_inputs(4, M, N, d)
    O, Od, lse, _ = orc.attn_jvp_fwd_head(Q, K, V, Qd, Kd, Vd)
    O2, Od2 = scalar_forward(*(x.tolist() for x in (Q, K, V, Qd, Kd, Vd)))
    assert np.allclose(O, np.array(O2), rtol=1e-13, atol=1e-13)
    assert np.allclose(Od, np.array(Od2), rtol=1e-12, atol=1e-12)


def test_two_key_closed_form():
    """One query, two keys, d = 1 (alpha = 1).  With D = q (k1 - k2): P1 = sigmoid(D),
    O = v2 + P1 (v1 - v2),  Odot = P1 P2 Ddot (v1 - v2) + P1 vd1 + P2 vd2,
    Ddot = qd (k1 - k2) + q (kd1 - kd2).  k1 - k2 = ln 3 gives P = (3/4, 1/4) exactly;
    gradients of L = g O + gd Odot follow by differentiating these two lines by hand.
    """
    ln3 = math.log(3.0)
    q, k1, k2, v1, v2 = 1.0, ln3, 0.0, 2.0, -2.0
    qd, kd1, kd2, vd1, vd2 = 1.0, 0.5, -0.5, 1.0, -1.0
    g, gd = 1.0, 2.0
    P1, P2 = 0.75, 0.25
    Dd = qd * (k1 - k2) + q * (kd1 - kd2)
    dv = v1 - v2
    O_exp = v2 + P1 * dv
    Od_exp = P1 * P2 * Dd * dv + P1 * vd1 + P2 * vd2
    dL_dD = g * P1 * P2 * dv + gd * (P1 * P2 * (1 - 2 * P1) * Dd * dv + P1 * P2 * (vd1 - vd2))
    exp = dict(
        dq=dL_dD * (k1 - k2) + gd * P1 * P2 * dv * (kd1 - kd2),
        dk1=dL_dD * q + gd * P1 * P2 * dv * qd,
        dv1=g * P1 + gd * P1 * P2 * Dd, dv2=g * P2 - gd * P1 * P2 * Dd,
        dqd=gd * P1 * P2 * dv * (k1 - k2), dkd1=gd * P1 * P2 * dv * q,
        dvd1=gd * P1, dvd2=gd * P2)
    A = lambda *x: np.array(x, dtype=np.float64).reshape(-1, 1)
    O, Od, lse, mubar = orc.attn_jvp_fwd_head(A(q), A(k1, k2), A(v1, v2), A(qd), A(kd1, kd2), A(vd1, vd2))
    assert abs(O[0, 0] - O_exp) < 1e-14 and abs(O_exp - 1.0) < 1e-15
    assert abs(Od[0, 0] - Od_exp) < 1e-14
    assert abs(lse[0] - math.log(4.0)) < 1e-14
    assert abs(mubar[0] - (P1 * (ln3 + 0.5) + P2 * (-0.5))) < 1e-14
    dQ, dK, dV, dQd, dKd, dVd = orc.attn_jvp_bwd_head(
        A(q), A(k1, k2), A(v1, v2), A(qd), A(kd1, kd2), A(vd1, vd2), A(g), A(gd))
    assert abs(dQ[0, 0] - exp["dq"]) < 1e-13
    assert abs(dK[0, 0] - exp["dk1"]) < 1e-13 and abs(dK[1, 0] + exp["dk1"]) < 1e-13
    assert abs(dV[0, 0] - exp["dv1"]) < 1e-13 and abs(dV[1, 0] - exp["dv2"]) < 1e-13
    assert abs(dQd[0, 0] - exp["dqd"]) < 1e-13
    assert abs(dKd[0, 0] - exp["dkd1"]) < 1e-13 and abs(dKd[1, 0] + exp["dkd1"]) < 1e-13
    assert abs(dVd[0, 0] - exp["dvd1"]) < 1e-13 and abs(dVd[1, 0] - exp["dvd2"]) < 1e-13


# ----------------------------------------------------------------------------
# 3. an independent mechanism: PyTorch CPU float64 attention, forward-mode JVP and autograd
# ----------------------------------------------------------------------------
def torch_math_attention(q, k, v):
    s = (q @ k.transpose(-1, -2)) / math.sqrt(q.shape[-1])
    return torch.softmax(s, dim=-1) @ v


def test_against_torch_sdpa_jvp_autograd():
    B, H, N, d = 2, 3, 17, 8
    r = np.random.default_rng(5)
    arrs = [r.standard_normal((B, H, N, d)) for _ in range(8)]
    q, k, v, tq, tk, tv, gO, gTO = arrs
    o, to, lse, mubar = orc.attn_jvp_fwd(q, k, v, tq, tk, tv)
    grads = orc.attn_jvp_bwd(q, k, v, tq, tk, tv, gO, gTO)

    T = [torch.from_numpy(a).clone().requires_grad_(i < 6) for i, a in enumerate(arrs)]
    # library routine for the primal
    o_lib = torch.nn.functional.scaled_dot_product_attention(T[0], T[1], T[2])
    assert np.allclose(o, o_lib.detach().numpy(), rtol=1e-12, atol=1e-12)
    # forward-mode JVP of explicit-math attention (the construction of the paper's Fig. "JVP code")
    o_t, to_t = torch.func.jvp(torch_math_attention, (T[0], T[1], T[2]), (T[3], T[4], T[5]))
    assert np.allclose(to, to_t.detach().numpy(), rtol=1e-11, atol=1e-11)
    s = (T[0] @ T[1].transpose(-1, -2)) / math.sqrt(d)
    assert np.allclose(lse, torch.logsumexp(s, -1).detach().numpy(), rtol=1e-12, atol=1e-12)
    # reverse mode through both outputs
    L = (o_t * T[6]).sum() + (to_t * T[7]).sum()
    tg = torch.autograd.grad(L, T[:6])
    for mine, ref, name in zip(grads, tg, ("dq", "dk", "dv", "dtq", "dtk", "dtv")):
        assert np.allclose(mine, ref.numpy(), rtol=1e-10, atol=1e-10), name


# ----------------------------------------------------------------------------
# 4. the paper's Step 1-6 closed forms for the gTO path (gO = 0)
# ----------------------------------------------------------------------------
def paper_steps_gTO_path(Q, K, V, Qd, Kd, Vd, dOd):
    """App. C, Steps 1-6, as printed (Step 6's dV summed over i; Q_{i,:} in Step 4)."""
    d = Q.shape[1]
    a = 1.0 / math.sqrt(d)
    S = Q @ K.T
    Sd = Qd @ K.T + Q @ Kd.T
    m = (a * S).max(axis=1, keepdims=True)
    l = np.exp(a * S - m).sum(axis=1, keepdims=True)        # un-normalised sum
    ell = m + np.log(l)
    P = np.exp(a * S - ell)
    mu_over_l = (P * (a * Sd)).sum(axis=1, keepdims=True)
    Nm = a * Sd - mu_over_l
    E = dOd @ V.T
    F = dOd @ Vd.T
    Sig1 = (P * E).sum(axis=1, keepdims=True)
    Sig2 = (P * (F + E * Nm)).sum(axis=1, keepdims=True)
    W = (E - Sig1) * P
    dK1 = a * W.T @ Qd
    dKd = a * W.T @ Q
    dQ1 = a * W @ Kd
    dQd = a * W @ K
    X = (a * (-Sig1) * Sd + Sig1 * mu_over_l) * P + (F + E * (a * Sd - mu_over_l) - Sig2) * P
    dK = dK1 + a * X.T @ Q
    dQ = dQ1 + a * X @ K
    dVd = P.T @ dOd
    dV = (P * (a * Sd - mu_over_l)).T @ dOd
    return dQ, dK, dV, dQd, dKd, dVd


def test_paper_closed_forms_match_reverse_sweep():
    Q, K, V, Qd, Kd, Vd, _, Gd = head_inputs(6, 9, 11, 5)
    ref = paper_steps_gTO_path(Q, K, V, Qd, Kd, Vd, Gd)
    got = orc.attn_jvp_bwd_head(Q, K, V, Qd, Kd, Vd, np.zeros_like(Gd), Gd)
    for a, b in zip(got, ref):
        assert np.allclose(a, b, rtol=1e-12, atol=1e-12)


def test_gTO_zero_is_ordinary_attention_backward():
    """gTO = 0: textbook softmax-attention backward dV = P^T G, dS = P o (G V^T - rowsum(G o O))."""
    Q, K, V, Qd, Kd, Vd, G, _ = head_inputs(8, 7, 10, 4)
    a = 0.5
    z = a * Q @ K.T
    P = np.exp(z - z.max(1, keepdims=True))
    P /= P.sum(1, keepdims=True)
    O = P @ V
    dS = P * (G @ V.T - (G * O).sum(1, keepdims=True))
    got = orc.attn_jvp_bwd_head(Q, K, V, Qd, Kd, Vd, G, np.zeros_like(G))
    assert np.allclose(got[0], a * dS @ K, atol=1e-13)
    assert np.allclose(got[1], a * dS.T @ Q, atol=1e-13)
    assert np.allclose(got[2], P.T @ G, atol=1e-13)
    for g in got[3:]:
        assert np.abs(g).max() == 0.0


# ----------------------------------------------------------------------------
# 5. invariants and special cases
# ----------------------------------------------------------------------------
def test_softmax_rows_sum_to_one_via_constant_values():
    Q, K, V, Qd, Kd, Vd, _, _ = head_inputs(9, 5, 8, 3)
    ones = np.ones_like(V)
    O, Od, _, _ = orc.attn_jvp_fwd_head(Q, K, ones, Qd, Kd, np.zeros_like(V))
    assert np.allclose(O, 1.0, atol=1e-14)          # P 1 = 1
    assert np.abs(Od).max() < 1e-14                 # (P o N) 1 = mubar - mubar = 0


def test_zero_tangents_give_zero():
    Q, K, V, *_ = head_inputs(10, 5, 8, 3)
    Z = np.zeros_like
    _, Od, _, mubar = orc.attn_jvp_fwd_head(Q, K, V, Z(Q), Z(K), Z(V))
    assert np.abs(Od).max() == 0.0 and np.abs(mubar).max() == 0.0


def test_tangent_is_linear_in_tangents():
    Q, K, V, Qd, Kd, Vd, _, _ = head_inputs(11, 6, 6, 4)
    Q2, K2, V2 = rnd(12, 6, 4), rnd(13, 6, 4), rnd(14, 6, 4)
    f = lambda a, b, c: orc.attn_jvp_fwd_head(Q, K, V, a, b, c)[1]
    lhs = f(2.0 * Qd - 3.0 * Q2, 2.0 * Kd - 3.0 * K2, 2.0 * Vd - 3.0 * V2)
    rhs = 2.0 * f(Qd, Kd, Vd) - 3.0 * f(Q2, K2, V2)
    assert np.allclose(lhs, rhs, atol=1e-12)


def test_only_value_tangent_is_attention_of_value_tangent():
    Q, K, V, _, _, Vd, _, _ = head_inputs(15, 5, 9, 4)
    Z = np.zeros_like
    O, Od, _, _ = orc.attn_jvp_fwd_head(Q, K, V, Z(Q), Z(K), Vd)
    assert np.allclose(Od, plain_attention(Q, K, Vd, 0.5), atol=1e-14)
    O2, Od2, _, _ = orc.attn_jvp_fwd_head(Q, K, V, Z(Q), Z(K), V)
    assert np.allclose(Od2, O2, atol=1e-14)


def test_constant_key_tangent_is_shift_invariant():
    """Kdot_j = u for all j, Qdot = 0: Sdot_ij = Q_i.u is constant along a row, so N = 0."""
    Q, K, V, _, _, Vd, _, _ = head_inputs(16, 5, 9, 4)
    u = rnd(17, 1, 4)
    O, Od, _, _ = orc.attn_jvp_fwd_head(Q, K, V, np.zeros_like(Q), np.repeat(u, 9, 0), Vd)
    assert np.allclose(Od, plain_attention(Q, K, Vd, 0.5), atol=1e-13)


def test_single_key():
    Q, K, V, Qd, Kd, Vd, G, Gd = head_inputs(18, 4, 1, 3)
    O, Od, lse, _ = orc.attn_jvp_fwd_head(Q, K, V, Qd, Kd, Vd)
    assert np.allclose(O, np.repeat(V, 4, 0)) and np.allclose(Od, np.repeat(Vd, 4, 0))
    dQ, dK, dV, dQd, dKd, dVd = orc.attn_jvp_bwd_head(Q, K, V, Qd, Kd, Vd, G, Gd)
    assert np.allclose(dV, G.sum(0, keepdims=True)) and np.allclose(dVd, Gd.sum(0, keepdims=True))
    for g in (dQ, dK, dQd, dKd):
        assert np.abs(g).max() < 1e-14


def test_zero_queries_uniform_softmax():
    _, K, V, Qd, Kd, Vd, _, _ = head_inputs(19, 4, 6, 2)
    Q = np.zeros((4, 2))
    O, Od, lse, _ = orc.attn_jvp_fwd_head(Q, K, V, Qd, Kd, Vd)
    assert np.allclose(O, V.mean(0, keepdims=True).repeat(4, 0), atol=1e-14)
    assert np.allclose(lse, math.log(6.0), atol=1e-14)
    zd = (Qd @ K.T) / math.sqrt(2.0)
    exp = Vd.mean(0, keepdims=True) + ((zd - zd.mean(1, keepdims=True)) @ V) / 6.0
    assert np.allclose(Od, exp, atol=1e-13)


def test_key_gradients_sum_to_zero_over_keys():
    """Adding one vector to every key changes neither O nor Odot (softmax shift), so
    sum_j dK_j = 0; adding one vector to every Kdot_j leaves Odot unchanged, so sum_j dKdot_j = 0."""
    args = head_inputs(20, 7, 9, 4)
    _, dK, _, _, dKd, _ = orc.attn_jvp_bwd_head(*args)
    assert np.abs(dK.sum(0)).max() < 1e-12 and np.abs(dKd.sum(0)).max() < 1e-12


def test_row_sums_two_forms_agree():
    """Sigma_1 = rowsum(P o (gTO V^T)) = rowsum(gTO o O);  the paper's Sigma_2 = rowsum(gTO o Odot)."""
    Q, K, V, Qd, Kd, Vd, _, Gd = head_inputs(21, 6, 8, 3)
    a = 1.0 / math.sqrt(3)
    O, Od, lse, mubar = orc.attn_jvp_fwd_head(Q, K, V, Qd, Kd, Vd)
    P = np.exp(a * Q @ K.T - lse[:, None])
    Nm = a * (Qd @ K.T + Q @ Kd.T) - mubar[:, None]
    E, F = Gd @ V.T, Gd @ Vd.T
    assert np.allclose((P * E).sum(1), (Gd * O).sum(1), atol=1e-13)
    assert np.allclose((P * (F + E * Nm)).sum(1), (Gd * Od).sum(1), atol=1e-13)


def test_explicit_scale_and_batched_wrapper():
    r = np.random.default_rng(22)
    arrs = [r.standard_normal((2, 2, 5, 3)) for _ in range(8)]
    o, to, lse, mubar = orc.attn_jvp_fwd(*arrs[:6], scale=0.37)
    o2, to2, lse2, mubar2 = orc.attn_jvp_fwd_head(*(a[1, 0] for a in arrs[:6]), scale=0.37)
    assert np.array_equal(o[1, 0], o2) and np.array_equal(to[1, 0], to2)
    assert np.allclose(o2, plain_attention(arrs[0][1, 0], arrs[1][1, 0], arrs[2][1, 0], 0.37), atol=1e-14)
    g = orc.attn_jvp_bwd(*arrs, scale=0.37)
    g2 = orc.attn_jvp_bwd_head(*(a[0, 1] for a in arrs), scale=0.37)
    for x, y in zip(g, g2):
        assert np.array_equal(x[0, 1], y)


def test_query_rows_are_independent():
    """A query row's outputs depend on no other query row, and the key-side gradients are sums over
    the query rows: the oracle applied to blocks of query rows (M != N, which its definition allows)
    gives the whole-head result.  The long-sequence GPU tests lean on this."""
    args = head_inputs(23, 11, 11, 4)
    Q, K, V, Qd, Kd, Vd, G, Gd = args
    whole_f = orc.attn_jvp_fwd_head(*args[:6])
    whole_g = orc.attn_jvp_bwd_head(*args)
    dK, dV, dKd, dVd = (np.zeros_like(K) for _ in range(4))
    for r in (slice(0, 4), slice(4, 5), slice(5, 11)):
        f = orc.attn_jvp_fwd_head(Q[r], K, V, Qd[r], Kd, Vd)
        for x, y in zip(f, whole_f):
            assert np.allclose(x, y[r], atol=1e-14)
        g = orc.attn_jvp_bwd_head(Q[r], K, V, Qd[r], Kd, Vd, G[r], Gd[r])
        assert np.allclose(g[0], whole_g[0][r], atol=1e-13) and np.allclose(g[3], whole_g[3][r], atol=1e-13)
        dK += g[1]
        dV += g[2]
        dKd += g[4]
        dVd += g[5]
    for x, y in zip((dK, dV, dKd, dVd), (whole_g[1], whole_g[2], whole_g[4], whole_g[5])):
        assert np.allclose(x, y, atol=1e-13)
