"""Float64 CPU oracle for the normalised adaptive-layer-norm modulation, its JVP tangent and its backward.

TEST INFRASTRUCTURE ONLY.  Imported by tests/ and nothing else; it shares no code with the HIP kernels and
never calls them.

What it follows (Terminal Velocity Matching, Sec. "Semi-Lipschitz control", the equation for AdaLN(x, t), and
App. "Full Description of Normalization of Modulation"): with RMSNorm^- the RMSNorm without learnable
parameters,

    AdaLN(x, t) = RMSNorm^-(x) o RMSNorm^-(a(t)) + RMSNorm^-(b(t)),

x a token's features (C of them), a(t) and b(t) the scale and shift that the time embedding produces for the
token's batch element, each normalised over its C entries.  (This is the operand of ATTN and of MLP in the
appendix's layer equations.)  All three inputs carry tangents: the network's JVP runs along the time argument,
which moves x, a and b.  RMSNorm^- itself is taken from rmsnorm_oracle with a unit gain: mean of squares,
eps inside the square root (see that module's header for the reading of the printed formula).

The tangent is the directional derivative along (tx, ta, tb) by the product rule; the backward is the
gradient of <gy, y> + <gty, ty> with respect to x, tx, a, ta, b, tb, as a reverse sweep over the three
normalisations and the product, the gradients of a and b summed over the tokens of their batch element.

Pins (tests/test_adaln_oracle.py): central finite differences of the plain definition for the tangent and for
every gradient; torch's rms_norm under torch.func.jvp and autograd in float64; special cases (constant a makes
the scale a vector of ones or minus ones; zero tangents; one token per batch element).
"""
import numpy as np

from oracle import rmsnorm_oracle as rn


def adaln_jvp_fwd(x, tx, a, ta, b, tb, eps):
    """x, tx: [B, T, C]; a, ta, b, tb: [B, C].  Returns (y, ty), [B, T, C]."""
    x, tx, a, ta, b, tb = (np.asarray(v, dtype=np.float64) for v in (x, tx, a, ta, b, tb))
    one = np.ones(x.shape[-1])
    xh, txh = rn.rmsnorm_jvp_fwd(x, tx, one, eps)
    ah, tah = rn.rmsnorm_jvp_fwd(a, ta, one, eps)
    bh, tbh = rn.rmsnorm_jvp_fwd(b, tb, one, eps)
    y = xh * ah[:, None, :] + bh[:, None, :]
    ty = txh * ah[:, None, :] + xh * tah[:, None, :] + tbh[:, None, :]
    return y, ty


def adaln_jvp_bwd(x, tx, a, ta, b, tb, eps, gy, gty):
    """Gradient of <gy, y> + <gty, ty>.  Returns (gx, gtx, ga, gta, gb, gtb)."""
    x, tx, a, ta, b, tb, gy, gty = (np.asarray(v, dtype=np.float64) for v in (x, tx, a, ta, b, tb, gy, gty))
    one = np.ones(x.shape[-1])
    xh, txh = rn.rmsnorm_jvp_fwd(x, tx, one, eps)
    ah, tah = rn.rmsnorm_jvp_fwd(a, ta, one, eps)
    # through y = xh ah + bh and ty = txh ah + xh tah + tbh
    g_xh = gy * ah[:, None, :] + gty * tah[:, None, :]
    g_txh = gty * ah[:, None, :]
    g_ah = np.sum(gy * xh + gty * txh, axis=1)
    g_tah = np.sum(gty * xh, axis=1)
    g_bh = np.sum(gy, axis=1)
    g_tbh = np.sum(gty, axis=1)
    # through the three normalisations (unit gain; its gradient is not wanted)
    gx, gtx, _ = rn.rmsnorm_jvp_bwd(x, tx, one, eps, g_xh, g_txh)
    ga, gta, _ = rn.rmsnorm_jvp_bwd(a, ta, one, eps, g_ah, g_tah)
    gb, gtb, _ = rn.rmsnorm_jvp_bwd(b, tb, one, eps, g_bh, g_tbh)
    return gx, gtx, ga, gta, gb, gtb
