"""Float64 CPU oracle for softmax attention with a JVP tangent, and its backward.

TEST INFRASTRUCTURE ONLY.  This module is the slow, dense, obviously-correct
statement of what the GPU library computes.  It is imported by tests/, by
__graft_entry__.smoke() and by bench.py's cpu_baseline leg, and by nothing
else; it shares no code with the HIP path and never calls it.

What it follows (Terminal Velocity Matching, App. C "Flash Attention JVP with
Backward Pass"):

  * Eq. (sdpa) with the "Background" paragraph: per head, queries Q [M,d],
    keys K [N,d], values V [N,d], alpha = 1/sqrt(d),
    O = softmax_rows(alpha Q K^T) V.  (The equation prints V in front of the
    softmax; the shapes only admit softmax(.) V.)
  * The un-numbered equations under "Step 1": S = Q K^T,
    Sdot = Qdot K^T + Q Kdot^T, P = exp(alpha S - lse), mu/l = sum_j P (alpha Sdot),
    N = alpha Sdot - mu/l.  The tangent output is the directional derivative of
    eq. (sdpa) along (Qdot, Kdot, Vdot):  Odot = (P o N) V + P Vdot.
  * "Caching softmax statistics": per query row the log-sum-exp (natural log,
    of the scaled scores) and the ratio mu/l (called `mubar` here; only the
    ratio ever enters a later formula).
  * Backward: the gradient of  L = <gO, O> + <gTO, Odot>  with respect to all
    six inputs.  The paper gives closed forms for the gTO path in Steps 1-6 and
    delegates the gO path to ordinary attention backward; this oracle does not
    use those closed forms.  It runs a plain reverse sweep over the forward
    graph, node by node (generic softmax Jacobian included), so that the GPU
    kernels, which use the simplified closed forms, are an independent
    derivation of the same numbers.

Every N x N matrix is materialised; there is no tiling, fusion or reordering.
Matrix products are numpy matmuls in float64.

Pins (tests/test_oracle_*.py): central finite differences of eq. (sdpa) for the
tangent and of L for every gradient; a pure-Python scalar-loop evaluation on
tiny inputs; the closed-form 2-key / 1-dim case in tests/golden/; PyTorch's CPU
scaled_dot_product_attention, torch.func.jvp and autograd in float64 as an
independent mechanism; the paper's Step 1-6 closed forms for the gTO path;
invariants (rows of P sum to one, zero tangents, linearity, shift invariance,
column sums of dK and dKdot vanish) and special cases (N = 1, Q = 0,
Qdot = Kdot = 0).
"""
import numpy as np

__all__ = ["attn_jvp_fwd", "attn_jvp_bwd", "attn_jvp_fwd_head", "attn_jvp_bwd_head"]


def _alpha(d, scale):
    return (1.0 / np.sqrt(float(d))) if (scale is None or scale == 0.0) else float(scale)


def _softmax_rows(z):
    """Row softmax and row log-sum-exp of z [M,N] (stabilised by the row max)."""
    m = z.max(axis=1, keepdims=True)
    e = np.exp(z - m)
    l = e.sum(axis=1, keepdims=True)
    return e / l, (m + np.log(l))[:, 0]


def attn_jvp_fwd_head(Q, K, V, Qd, Kd, Vd, scale=None):
    """One head.  Q,Qd [M,d]; K,V,Kd,Vd [N,d] float64.

    Returns O [M,d], Odot [M,d], lse [M], mubar [M]  (eq. (sdpa); equations
    under "Step 1"; "Caching softmax statistics").
    """
    a = _alpha(Q.shape[1], scale)
    z = a * (Q @ K.T)                       # alpha S
    zd = a * (Qd @ K.T + Q @ Kd.T)          # alpha Sdot
    P, lse = _softmax_rows(z)               # P_ij = exp(alpha S_ij - lse_i)
    mubar = (P * zd).sum(axis=1)            # mu_i / l_i
    Nm = zd - mubar[:, None]                # N_ij
    O = P @ V
    Od = (P * Nm) @ V + P @ Vd
    return O, Od, lse, mubar


def attn_jvp_bwd_head(Q, K, V, Qd, Kd, Vd, G, Gd, scale=None):
    """One head.  Gradient of L = <G,O> + <Gd,Odot> w.r.t. Q,K,V,Qd,Kd,Vd.

    Plain reverse sweep over the forward graph
        z = a Q K^T -> P = softmax(z);  zd = a (Qd K^T + Q Kd^T);
        mubar = rowsum(P o zd);  Nm = zd - mubar;  Pd = P o Nm;
        O = P V;  Odot = Pd V + P Vd.
    Returns dQ, dK, dV, dQd, dKd, dVd.
    """
    a = _alpha(Q.shape[1], scale)
    z = a * (Q @ K.T)
    zd = a * (Qd @ K.T + Q @ Kd.T)
    P, _ = _softmax_rows(z)
    mubar = (P * zd).sum(axis=1, keepdims=True)
    Nm = zd - mubar
    Pd = P * Nm

    # O = P V ; Odot = Pd V + P Vd
    dV = P.T @ G + Pd.T @ Gd
    dVd = P.T @ Gd
    gP = G @ V.T + Gd @ Vd.T
    gPd = Gd @ V.T
    # Pd = P o Nm
    gP = gP + gPd * Nm
    gNm = gPd * P
    # Nm = zd - mubar 1^T
    gzd = gNm.copy()
    gmubar = -gNm.sum(axis=1, keepdims=True)
    # mubar = rowsum(P o zd)
    gP = gP + gmubar * zd
    gzd = gzd + gmubar * P
    # P = softmax_rows(z): generic softmax Jacobian
    gz = P * (gP - (P * gP).sum(axis=1, keepdims=True))
    # z = a Q K^T ; zd = a (Qd K^T + Q Kd^T)
    dQ = a * (gz @ K + gzd @ Kd)
    dK = a * (gz.T @ Q + gzd.T @ Qd)
    dQd = a * (gzd @ K)
    dKd = a * (gzd.T @ Q)
    return dQ, dK, dV, dQd, dKd, dVd


def _as64(*xs):
    return [np.ascontiguousarray(np.asarray(x, dtype=np.float64)) for x in xs]


def attn_jvp_fwd(q, k, v, tq, tk, tv, scale=None):
    """Batched forward.  All inputs [B,H,N,d].  Returns o, to [B,H,N,d]; lse, mubar [B,H,N]."""
    q, k, v, tq, tk, tv = _as64(q, k, v, tq, tk, tv)
    B, H, M, d = q.shape
    o = np.empty_like(q)
    to = np.empty_like(q)
    lse = np.empty((B, H, M))
    mubar = np.empty((B, H, M))
    for b in range(B):
        for h in range(H):
            o[b, h], to[b, h], lse[b, h], mubar[b, h] = attn_jvp_fwd_head(
                q[b, h], k[b, h], v[b, h], tq[b, h], tk[b, h], tv[b, h], scale)
    return o, to, lse, mubar


def attn_jvp_bwd(q, k, v, tq, tk, tv, gO, gTO, scale=None):
    """Batched backward.  Returns dq, dk, dv, dtq, dtk, dtv, each [B,H,N,d]."""
    q, k, v, tq, tk, tv, gO, gTO = _as64(q, k, v, tq, tk, tv, gO, gTO)
    B, H = q.shape[:2]
    outs = [np.empty_like(x) for x in (q, k, v, q, k, v)]
    for b in range(B):
        for h in range(H):
            r = attn_jvp_bwd_head(q[b, h], k[b, h], v[b, h], tq[b, h], tk[b, h], tv[b, h],
                                  gO[b, h], gTO[b, h], scale)
            for dst, src in zip(outs, r):
                dst[b, h] = src
    return tuple(outs)
