"""Float64 CPU oracle for a linear layer applied to a token and to its JVP tangent, and its backward.

TEST INFRASTRUCTURE ONLY.  Imported by tests/ and nothing else; it shares no code with the HIP kernels and
never calls them.

What it follows (Terminal Velocity Matching, Sec. 4: the training objective differentiates through a
Jacobian-vector product of the whole network along its inputs (x_t, t, s); App. "Full Description of
Normalization of Modulation", the two layer equations, whose ATTN and MLP are built from linear layers: the
query/key/value and output projections around the attention, and the two layers around the MLP's activation).
A linear layer with weight W [F, K] and bias b [F] maps a token's features x [K] to

    y = W x + b,

and since the JVP runs along the network's inputs, not its parameters, W and b carry no tangent: the tangent of
y along the tangent tx of x is

    ty = W tx.

The backward is the gradient of  L = <gy, y> + <gty, ty>  with respect to x, tx, W and b, as a reverse sweep over
the two products (both outputs use the same W, so its gradient collects both):

    gx = W^T gy        gtx = W^T gty        gW = sum over tokens of (gy x^T + gty tx^T)        gb = sum over tokens of gy.

Tokens are the rows of x [R, K]; products are numpy matmuls in float64.

Pins (tests/test_linear_oracle.py): central finite differences of the plain map for the tangent and for every
gradient entry; torch.nn.functional.linear under torch.func.jvp and autograd in float64; scalar loops; special
cases (identity weight, zero tangent, one token and one feature by hand); linearity; planted mistakes.
"""
import numpy as np


def linear_jvp_fwd(x, tx, w, b=None):
    """x, tx: [R, K]; w: [F, K]; b: [F] or None.  Returns (y, ty), [R, F]."""
    x, tx, w = (np.asarray(v, dtype=np.float64) for v in (x, tx, w))
    y = x @ w.T
    if b is not None:
        y = y + np.asarray(b, dtype=np.float64)[None, :]
    ty = tx @ w.T
    return y, ty


def linear_jvp_bwd(x, tx, w, gy, gty):
    """Gradient of <gy, y> + <gty, ty>.  Returns (gx, gtx, gw, gb): [R, K], [R, K], [F, K], [F]."""
    x, tx, w, gy, gty = (np.asarray(v, dtype=np.float64) for v in (x, tx, w, gy, gty))
    # through ty = tx W^T
    gtx = gty @ w
    gw = gty.T @ tx
    # through y = x W^T + b
    gx = gy @ w
    gw = gw + gy.T @ x
    gb = gy.sum(axis=0)
    return gx, gtx, gw, gb
