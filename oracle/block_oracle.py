"""Float64 CPU oracle for one normalised DiT block with a JVP tangent, and its backward: the composition of the
per-operation oracles in this folder, nothing else.

TEST INFRASTRUCTURE ONLY.  Imported by tests/ and nothing else; it shares no code with the HIP kernels and
never calls them.

What it follows (Terminal Velocity Matching, App. "Full Description of Normalization of Modulation"): with the six
modulation vectors a1, b1, c1, a2, b2, c2 of a layer (each [B, C], each normalised by RMSNorm^-), the layer is

    x <- x + c1^- * ATTN( RMSNorm^-(x) * a1^- + b1^- )
    x <- x + c2^- * MLP ( RMSNorm^-(x) * a2^- + b2^- )

ATTN is multi-head attention as in DiT (Sec. "Semi-Lipschitz control": RMSNorm with a learnable gain as QK-norm):
one linear layer to q, k, v (split as [3, H, d] along the features), RMSNorm with gain over the head dimension of q
and of k, softmax attention per head (eq. (sdpa)), heads merged, one output linear layer.  MLP is linear, the
activation (tanh-form GELU, DiT's; the paper does not name it), linear.  The JVP of Sec. 4 runs along the network's
inputs: the stream x and all six modulation vectors carry tangents, the parameters do not.

Forward: every operation's oracle applied to (value, tangent) in the order above.  Backward: the gradient of
<gz, z> + <gtz, tz> (z, tz the block's outputs) by calling the operations' backward oracles in reverse order; where
the stream branches (into a modulation and along the residual connection) its two gradients are added.

Pins (tests/test_block_oracle.py): the same block written with torch's own linear, rms_norm,
softmax, matmul and gelu under torch.func.jvp and autograd in float64 (outputs and every gradient);
central finite differences of the forward for the tangent; planted mistakes in the wiring.
"""
import numpy as np

from oracle import adaln_oracle, gate_oracle, gelu_oracle, linear_oracle, rmsnorm_oracle, tvmattn_oracle

MODS = ("a1", "b1", "c1", "a2", "b2", "c2")
PARAMS = ("wqkv", "bqkv", "gq", "gk", "wo", "bo", "w1", "b1", "w2", "b2")


def _split_heads(y, H):
    """[B, T, 3C] -> three [B, H, T, d] (features split as [3, H, d])."""
    B, T, C3 = y.shape
    d = C3 // (3 * H)
    y5 = y.reshape(B, T, 3, H, d)
    return tuple(np.ascontiguousarray(y5[:, :, i].transpose(0, 2, 1, 3)) for i in range(3))


def _merge_heads(o):
    """[B, H, T, d] -> [B, T, H d]."""
    B, H, T, d = o.shape
    return np.ascontiguousarray(o.transpose(0, 2, 1, 3)).reshape(B, T, H * d)


def _merge_qkv(q, k, v):
    """Three [B, H, T, d] -> [B, T, 3C]: the inverse of _split_heads."""
    B, H, T, d = q.shape
    y5 = np.stack([t.transpose(0, 2, 1, 3) for t in (q, k, v)], axis=2)   # [B, T, 3, H, d]
    return y5.reshape(B, T, 3 * H * d)


def _lin(x, tx, w, b):
    B, T, K = x.shape
    y, ty = linear_oracle.linear_jvp_fwd(x.reshape(B * T, K), tx.reshape(B * T, K), w, b)
    return y.reshape(B, T, -1), ty.reshape(B, T, -1)


def _lin_bwd(x, tx, w, gy, gty):
    B, T, K = x.shape
    F = w.shape[0]
    gx, gtx, gw, gb = linear_oracle.linear_jvp_bwd(x.reshape(B * T, K), tx.reshape(B * T, K), w, gy.reshape(B * T, F),
                                                   gty.reshape(B * T, F))
    return gx.reshape(B, T, K), gtx.reshape(B, T, K), gw, gb


def block_jvp_fwd(x, tx, mods, tmods, params, H, eps, qk_eps, keep=False):
    """x, tx: [B, T, C]; mods, tmods: dicts of the six [B, C] vectors and of their tangents; params: dict of wqkv
    [3C, C], bqkv [3C], gq, gk [d], wo [C, C], bo [C], w1 [F, C], b1 [F], w2 [C, F], b2 [C].  eps: of RMSNorm^-;
    qk_eps: of the QK-norm.  Returns (z, tz); with keep=True also the dict of intermediate (value, tangent) pairs."""
    f = lambda v: np.asarray(v, dtype=np.float64)
    x, tx = f(x), f(tx)
    m = {n: f(mods[n]) for n in MODS}
    tm = {n: f(tmods[n]) for n in MODS}
    p = {n: f(params[n]) for n in PARAMS}
    s = {}
    s["u1"] = adaln_oracle.adaln_jvp_fwd(x, tx, m["a1"], tm["a1"], m["b1"], tm["b1"], eps)
    s["qkv"] = _lin(*s["u1"], p["wqkv"], p["bqkv"])
    q, k, v = _split_heads(s["qkv"][0], H)
    tq, tk, tv = _split_heads(s["qkv"][1], H)
    s["q"], s["k"], s["v"] = (q, tq), (k, tk), (v, tv)
    s["qn"] = rmsnorm_oracle.rmsnorm_jvp_fwd(q, tq, p["gq"], qk_eps)
    s["kn"] = rmsnorm_oracle.rmsnorm_jvp_fwd(k, tk, p["gk"], qk_eps)
    o, to, _, _ = tvmattn_oracle.attn_jvp_fwd(s["qn"][0], s["kn"][0], v, s["qn"][1], s["kn"][1], tv)
    s["o"] = (_merge_heads(o), _merge_heads(to))
    s["h1"] = _lin(*s["o"], p["wo"], p["bo"])
    s["x1"] = gate_oracle.gate_jvp_fwd(x, tx, *s["h1"], m["c1"], tm["c1"], eps)
    s["u2"] = adaln_oracle.adaln_jvp_fwd(*s["x1"], m["a2"], tm["a2"], m["b2"], tm["b2"], eps)
    s["p"] = _lin(*s["u2"], p["w1"], p["b1"])
    s["act"] = gelu_oracle.gelu_jvp_fwd(*s["p"])
    s["h2"] = _lin(*s["act"], p["w2"], p["b2"])
    z, tz = gate_oracle.gate_jvp_fwd(*s["x1"], *s["h2"], m["c2"], tm["c2"], eps)
    return (z, tz, s) if keep else (z, tz)


def block_jvp_bwd(x, tx, mods, tmods, params, H, eps, qk_eps, gz, gtz):
    """Gradient of <gz, z> + <gtz, tz>.  Returns a dict: "x", "tx", the six modulation vectors (a1 ... c2) and their
    tangents ("ta1" ... "tc2"), and every parameter (wqkv ... b2)."""
    f = lambda v: np.asarray(v, dtype=np.float64)
    x, tx, gz, gtz = f(x), f(tx), f(gz), f(gtz)
    m = {n: f(mods[n]) for n in MODS}
    tm = {n: f(tmods[n]) for n in MODS}
    p = {n: f(params[n]) for n in PARAMS}
    _, _, s = block_jvp_fwd(x, tx, mods, tmods, params, H, eps, qk_eps, keep=True)
    g = {}
    # z = x1 + c2^- * h2
    gx1, gtx1, gh2, gth2, g["c2"], g["tc2"] = gate_oracle.gate_jvp_bwd(*s["x1"], *s["h2"], m["c2"], tm["c2"], eps, gz, gtz)
    gact, gtact, g["w2"], g["b2"] = _lin_bwd(*s["act"], p["w2"], gh2, gth2)
    gp, gtp = gelu_oracle.gelu_jvp_bwd(*s["p"], gact, gtact)
    gu2, gtu2, g["w1"], g["b1"] = _lin_bwd(*s["u2"], p["w1"], gp, gtp)
    ax, atx, g["a2"], g["ta2"], g["b2m"], g["tb2m"] = adaln_oracle.adaln_jvp_bwd(*s["x1"], m["a2"], tm["a2"], m["b2"],
                                                                              tm["b2"], eps, gu2, gtu2)
    gx1, gtx1 = gx1 + ax, gtx1 + atx          # the stream feeds the modulation and the residual connection
    # x1 = x + c1^- * h1
    gx, gtx, gh1, gth1, g["c1"], g["tc1"] = gate_oracle.gate_jvp_bwd(x, tx, *s["h1"], m["c1"], tm["c1"], eps, gx1, gtx1)
    go, gto, g["wo"], g["bo"] = _lin_bwd(*s["o"], p["wo"], gh1, gth1)
    B, T, C = x.shape
    d = C // H
    heads = lambda t: np.ascontiguousarray(t.reshape(B, T, H, d).transpose(0, 2, 1, 3))
    dqn, dkn, dv, dtqn, dtkn, dtv = tvmattn_oracle.attn_jvp_bwd(s["qn"][0], s["kn"][0], s["v"][0], s["qn"][1], s["kn"][1],
                                                                s["v"][1], heads(go), heads(gto))
    dq, dtq, g["gq"] = rmsnorm_oracle.rmsnorm_jvp_bwd(*s["q"], p["gq"], qk_eps, dqn, dtqn)
    dk, dtk, g["gk"] = rmsnorm_oracle.rmsnorm_jvp_bwd(*s["k"], p["gk"], qk_eps, dkn, dtkn)
    gqkv, gtqkv = _merge_qkv(dq, dk, dv), _merge_qkv(dtq, dtk, dtv)
    gu1, gtu1, g["wqkv"], g["bqkv"] = _lin_bwd(*s["u1"], p["wqkv"], gqkv, gtqkv)
    ax, atx, g["a1"], g["ta1"], g["b1m"], g["tb1m"] = adaln_oracle.adaln_jvp_bwd(x, tx, m["a1"], tm["a1"], m["b1"], tm["b1"],
                                                                              eps, gu1, gtu1)
    g["x"], g["tx"] = gx + ax, gtx + atx
    # (the modulation shifts b1, b2 share their names with the MLP's biases: the shifts are returned as "mb1", "mb2")
    out = {"x": g["x"], "tx": g["tx"]}
    for n in ("a1", "c1", "a2", "c2"):
        out[n], out["t" + n] = g[n], g["t" + n]
    out["mb1"], out["tmb1"], out["mb2"], out["tmb2"] = g["b1m"], g["tb1m"], g["b2m"], g["tb2m"]
    for n in PARAMS:
        out[n] = g[n]
    return out
