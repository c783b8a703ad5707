"""Float64 CPU oracle for RMSNorm with a learnable gain as QK-norm, its JVP tangent and its backward.

TEST INFRASTRUCTURE ONLY.  Imported by tests/ (and by bench.py's cpu_baseline leg, if it ever times it),
never by the product path; it shares no code with the HIP kernels and never calls them.

What it follows (Terminal Velocity Matching, Sec. "Semi-Lipschitz control" and App. "Lipschitzness of
RMSNorm"): the queries and keys that enter attention are normalised row by row,

    RMSNorm(x) = x / RMS(x),   RMS(x) = sqrt( (1/d) sum_i x_i^2 + eps ),

times a learnable gain g in R^d ("RMSNorm as QK-Norm ... with learnable scaling").  The appendix prints
the mean of x_i without the square; the name, and the Jacobian printed right under it
(delta_ij / RMS - x_i x_j / (d RMS^3)), are those of the mean of squares, which is what is taken here.
eps sits inside the square root, as printed.

The tangent is the directional derivative of y = g o x / RMS(x) along tx (the gain has no tangent: in the
paper's JVP only the network inputs carry one).  The backward is the gradient of <gy, y> + <gty, ty> with
respect to x, tx and g, by a plain reverse sweep over the forward graph, node by node; the GPU kernels use
the simplified closed form, an independent derivation of the same numbers.

Pins (tests/test_rmsnorm_oracle.py): the Jacobian the paper prints; central finite differences for the
tangent and for every gradient; torch's own rms_norm under torch.func.jvp and autograd in float64; the
closed-form two-element case in tests/golden/; invariants (scale invariance at eps = 0, so the tangent
along x vanishes and <gx, x> + <gtx, tx> = 0; unit RMS of y / g; linearity in tx).
"""
import numpy as np


def rmsnorm_jvp_fwd(x, tx, g, eps):
    """x, tx: [..., d]; g: [d].  Returns (y, ty)."""
    x, tx, g = (np.asarray(a, dtype=np.float64) for a in (x, tx, g))
    ms = np.mean(x * x, axis=-1, keepdims=True) + eps
    rms = np.sqrt(ms)
    y = g * (x / rms)
    # derivative of the quotient x / rms along tx; d(rms) = mean(x tx) / rms
    drms = np.mean(x * tx, axis=-1, keepdims=True) / rms
    ty = g * (tx / rms - x * drms / (rms * rms))
    return y, ty


def rmsnorm_jvp_bwd(x, tx, g, eps, gy, gty):
    """Gradient of <gy, y> + <gty, ty>.  Returns (gx, gtx, gg); gg is summed over all rows."""
    x, tx, g, gy, gty = (np.asarray(a, dtype=np.float64) for a in (x, tx, g, gy, gty))
    d = x.shape[-1]
    # forward graph, one node per line
    ms = np.mean(x * x, axis=-1, keepdims=True) + eps
    rms = np.sqrt(ms)
    inv = 1.0 / rms
    xh = x * inv            # y = g * xh
    c = np.mean(x * tx, axis=-1, keepdims=True)
    drms = c * inv
    a = tx * inv
    b = x * drms * inv * inv
    th = a - b              # ty = g * th
    # reverse sweep
    gg = np.sum((gy * xh + gty * th).reshape(-1, d), axis=0)
    g_xh = g * gy
    g_th = g * gty
    g_a = g_th
    g_b = -g_th
    g_x = np.zeros_like(x)
    g_tx = np.zeros_like(x)
    g_inv = np.zeros_like(inv)
    # a = tx * inv
    g_tx += g_a * inv
    g_inv += np.sum(g_a * tx, axis=-1, keepdims=True)
    # b = x * drms * inv^2
    g_x += g_b * drms * inv * inv
    g_drms = np.sum(g_b * x, axis=-1, keepdims=True) * inv * inv
    g_inv += np.sum(g_b * x, axis=-1, keepdims=True) * drms * 2.0 * inv
    # drms = c * inv
    g_c = g_drms * inv
    g_inv += g_drms * c
    # c = mean(x * tx)
    g_x += g_c * tx / d
    g_tx += g_c * x / d
    # xh = x * inv
    g_x += g_xh * inv
    g_inv += np.sum(g_xh * x, axis=-1, keepdims=True)
    # inv = 1 / rms, rms = sqrt(ms), ms = mean(x^2) + eps
    g_rms = -g_inv / (rms * rms)
    g_ms = g_rms / (2.0 * rms)
    g_x += g_ms * 2.0 * x / d
    return g_x, g_tx, gg
