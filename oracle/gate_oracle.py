"""Float64 CPU oracle for the normalised gate of a residual branch, its JVP tangent and its backward.

TEST INFRASTRUCTURE ONLY.  Imported by tests/ and nothing else; it shares no code with the HIP kernels and
never calls them.

What it follows (Terminal Velocity Matching, App. "Full Description of Normalization of Modulation", the two
layer equations): a block's branch output h (of ATTN or of MLP) re-enters the residual stream as

    z = x + RMSNorm^-(c(t)) o h,

x the stream's features of a token (C of them), h the branch output for that token, c(t) the gate that the
time embedding produces for the token's batch element, normalised over its C entries by RMSNorm^- (the RMSNorm
without learnable parameters).  All three inputs carry tangents: the network's JVP runs along the time
argument, which moves x, h and c.  RMSNorm^- itself is taken from rmsnorm_oracle with a unit gain: mean of
squares, eps inside the square root (see that module's header for the reading of the printed formula).

The tangent is the directional derivative along (tx, th, tc) by the product rule; the backward is the
gradient of <gz, z> + <gtz, tz> with respect to x, tx, h, th, c, tc, as a reverse sweep over the sum, the
product and the normalisation, the gradients of c summed over the tokens of its batch element.

Pins (tests/test_gate_oracle.py): central finite differences of the plain definition for the tangent and for
every gradient entry; torch's rms_norm under torch.func.jvp and autograd in float64; special cases (a constant
gate normalises to ones, so z = x + h; zero tangents; linearity; gradients of c as sums of one-token gradients).
"""
import numpy as np

from oracle import rmsnorm_oracle as rn


def gate_jvp_fwd(x, tx, h, th, c, tc, eps):
    """x, tx, h, th: [B, T, C]; c, tc: [B, C].  Returns (z, tz), [B, T, C]."""
    x, tx, h, th, c, tc = (np.asarray(v, dtype=np.float64) for v in (x, tx, h, th, c, tc))
    one = np.ones(x.shape[-1])
    ch, tch = rn.rmsnorm_jvp_fwd(c, tc, one, eps)
    z = x + ch[:, None, :] * h
    tz = tx + tch[:, None, :] * h + ch[:, None, :] * th
    return z, tz


def gate_jvp_bwd(x, tx, h, th, c, tc, eps, gz, gtz):
    """Gradient of <gz, z> + <gtz, tz>.  Returns (gx, gtx, gh, gth, gc, gtc)."""
    h, th, c, tc, gz, gtz = (np.asarray(v, dtype=np.float64) for v in (h, th, c, tc, gz, gtz))
    one = np.ones(h.shape[-1])
    ch, tch = rn.rmsnorm_jvp_fwd(c, tc, one, eps)
    # through z = x + ch h and tz = tx + tch h + ch th
    gx, gtx = gz.copy(), gtz.copy()
    gh = gz * ch[:, None, :] + gtz * tch[:, None, :]
    gth = gtz * ch[:, None, :]
    g_ch = np.sum(gz * h + gtz * th, axis=1)
    g_tch = np.sum(gtz * h, axis=1)
    # through the normalisation of the gate (unit gain; its gradient is not wanted)
    gc, gtc, _ = rn.rmsnorm_jvp_bwd(c, tc, one, eps, g_ch, g_tch)
    return gx, gtx, gh, gth, gc, gtc
