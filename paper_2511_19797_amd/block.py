"""One normalised DiT block with a JVP tangent, forward and backward, as a sequence of library calls.

The block of Terminal Velocity Matching, App. "Full Description of Normalization of Modulation":

    x <- x + c1^- * ATTN( RMSNorm^-(x) * a1^- + b1^- )        x <- x + c2^- * MLP( RMSNorm^-(x) * a2^- + b2^- )

with ATTN = linear to q, k, v -> RMSNorm with gain on q and k (QK-norm) -> attention -> linear, and MLP = linear ->
tanh-form GELU -> linear, every tensor carrying its tangent along the network's inputs (Sec. 4).  This module holds
no arithmetic: each step is one entry point of the binding, and the views between them are strides only:
q, k, v are the three slices of the fused projection's [B,T,3,H,d] output (the attention takes their strides), the
attention output is laid out like its queries and read by the output projection through a row pitch, and the
backward writes the gradients of q, k, v straight into the slices of one fused buffer for the projection's backward.
"""
import torch

from . import binding as tvm

MODS = ("a1", "b1", "c1", "a2", "b2", "c2")


def _heads(t5, i):
    """Slice i of a [B,T,3,H,d] buffer as a [B,H,T,d] view."""
    return t5[:, :, i].permute(0, 2, 1, 3)


def _rows(t_bhtd):
    """A [B,H,T,d] view laid out as [B,T,(gap),H,d] seen as rows [B*T, H*d] with its row pitch."""
    B, H, T, d = t_bhtd.shape
    return t_bhtd.permute(0, 2, 1, 3).reshape(B * T, H * d)


def block_jvp_fwd(x, tx, mods, tmods, params, H, eps, qk_eps):
    """x, tx: [B,T,C] bf16; mods, tmods: dicts of the six float32 [B,C] modulation vectors and their tangents; params:
    wqkv [3C,C], bqkv, wo [C,C], bo, w1 [F,C], b1, w2 [C,F], b2 (bf16) and the QK-norm gains gq, gk (float32 [d]).
    Returns (z, tz, saved): the block's output, its tangent, and what the backward needs."""
    B, T, C = x.shape
    d = C // H
    s = {}
    s["u1"] = tvm.tvmattn_adaln_jvp_fwd(x, tx, mods["a1"], tmods["a1"], mods["b1"], tmods["b1"], eps)
    qkv, tqkv = tvm.tvmattn_linear_jvp_fwd(*s["u1"], params["wqkv"], params["bqkv"])
    q5, tq5 = qkv.view(B, T, 3, H, d), tqkv.view(B, T, 3, H, d)
    s["q"], s["k"], s["v"] = ((_heads(q5, i), _heads(tq5, i)) for i in range(3))
    qn, tqn, kn, tkn = tvm.tvmattn_qknorm_jvp_fwd(s["q"][0], s["q"][1], s["k"][0], s["k"][1], params["gq"], params["gk"], qk_eps)
    s["qn"], s["kn"] = (qn, tqn), (kn, tkn)
    s["att"] = tvm.tvmattn_jvp_fwd(qn, kn, s["v"][0], tqn, tkn, s["v"][1])        # o, to, lse, stats; o laid out like qn
    s["o2d"] = (_rows(s["att"][0]), _rows(s["att"][1]))
    h1, th1 = tvm.tvmattn_linear_jvp_fwd(*s["o2d"], params["wo"], params["bo"])
    s["h1"] = (h1.view(B, T, C), th1.view(B, T, C))
    s["x1"] = tvm.tvmattn_gate_jvp_fwd(x, tx, *s["h1"], mods["c1"], tmods["c1"], eps)
    s["u2"] = tvm.tvmattn_adaln_jvp_fwd(*s["x1"], mods["a2"], tmods["a2"], mods["b2"], tmods["b2"], eps)
    s["p"] = tvm.tvmattn_linear_jvp_fwd(*s["u2"], params["w1"], params["b1"])
    s["act"] = tvm.tvmattn_gelu_jvp_fwd(*s["p"])
    s["h2"] = tvm.tvmattn_linear_jvp_fwd(*s["act"], params["w2"], params["b2"])
    z, tz = tvm.tvmattn_gate_jvp_fwd(*s["x1"], *s["h2"], mods["c2"], tmods["c2"], eps)
    return z, tz, s


def block_jvp_bwd(x, tx, mods, tmods, params, H, eps, qk_eps, saved, gz, gtz):
    """The gradient of <gz, z> + <gtz, tz>.  Returns a dict: "x", "tx"; the modulation vectors "a1", "mb1", "c1", "a2",
    "mb2", "c2" and their tangents ("ta1", "tmb1", ...); the parameters by their names."""
    B, T, C = x.shape
    d = C // H
    s, g = saved, {}
    gh2, gth2, g["c2"], g["tc2"] = tvm.tvmattn_gate_jvp_bwd(*s["h2"], mods["c2"], tmods["c2"], eps, gz, gtz)
    gact, gtact, g["w2"], g["b2"] = tvm.tvmattn_linear_jvp_bwd(*s["act"], params["w2"], gh2, gth2)
    gp, gtp = tvm.tvmattn_gelu_jvp_bwd(*s["p"], gact, gtact)
    gu2, gtu2, g["w1"], g["b1"] = tvm.tvmattn_linear_jvp_bwd(*s["u2"], params["w1"], gp, gtp)
    # the stream's gradient: along the residual connection (gz, gtz themselves) plus through the modulation
    gx1, gtx1, g["a2"], g["ta2"], g["mb2"], g["tmb2"] = tvm.tvmattn_adaln_jvp_bwd(
        *s["x1"], mods["a2"], tmods["a2"], mods["b2"], tmods["b2"], eps, gu2, gtu2, gres=gz, gtres=gtz)
    gh1, gth1, g["c1"], g["tc1"] = tvm.tvmattn_gate_jvp_bwd(*s["h1"], mods["c1"], tmods["c1"], eps, gx1, gtx1)
    go2d, gto2d, g["wo"], g["bo"] = tvm.tvmattn_linear_jvp_bwd(*s["o2d"], params["wo"], gh1.view(B * T, C), gth1.view(B * T, C))
    o = s["att"][0]
    as_heads = lambda t2d: torch.as_strided(t2d, o.shape, o.stride(), t2d.storage_offset())   # laid out like o
    gO, gTO = as_heads(go2d), as_heads(gto2d)
    gqkv = torch.empty(B, T, 3, H, d, dtype=x.dtype, device=x.device)
    gtqkv = torch.empty_like(gqkv)
    dq, dk, dv = (_heads(gqkv, i) for i in range(3))
    dtq, dtk, dtv = (_heads(gtqkv, i) for i in range(3))
    (q, tq), (k, tk), (v, tv), (qn, tqn), (kn, tkn) = s["q"], s["k"], s["v"], s["qn"], s["kn"]
    _, to, lse, stats = s["att"]
    if tvm.tvmattn_jvp_bwd_qknorm_workspace_bytes(q, k) > 0:   # the norm's backward inside the attention backward
        out = tvm.tvmattn_jvp_bwd_qknorm(q, tq, k, tk, params["gq"], params["gk"], qk_eps, qn, tqn, kn, tkn, v, tv, o, to, lse,
                                         stats, gO, gTO, out=(dq, dk, dv, dtq, dtk, dtv, torch.empty_like(params["gq"]),
                                                              torch.empty_like(params["gk"])))
        g["gq"], g["gk"] = out[6], out[7]
    else:
        dqn, dkn, _, dtqn, dtkn, _ = tvm.tvmattn_jvp_bwd(qn, kn, v, tqn, tkn, tv, o, to, lse, stats, gO, gTO,
                                                         out=(tvm._like(qn), tvm._like(kn), dv, tvm._like(qn), tvm._like(kn), dtv))
        out = tvm.tvmattn_qknorm_jvp_bwd(q, tq, k, tk, params["gq"], params["gk"], qk_eps, dqn, dtqn, dkn, dtkn,
                                         out=(dq, dtq, dk, dtk, torch.empty_like(params["gq"]), torch.empty_like(params["gk"])))
        g["gq"], g["gk"] = out[4], out[5]
    gu1, gtu1, g["wqkv"], g["bqkv"] = tvm.tvmattn_linear_jvp_bwd(*s["u1"], params["wqkv"], gqkv.view(B * T, 3 * C),
                                                                gtqkv.view(B * T, 3 * C))
    g["x"], g["tx"], g["a1"], g["ta1"], g["mb1"], g["tmb1"] = tvm.tvmattn_adaln_jvp_bwd(
        x, tx, mods["a1"], tmods["a1"], mods["b1"], tmods["b1"], eps, gu1, gtu1, gres=gx1, gtres=gtx1)
    return g
