"""Float64 CPU oracle for the MLP's pointwise activation with its JVP tangent and its backward.

TEST INFRASTRUCTURE ONLY.  Imported by tests/ and nothing else; it shares no code with the HIP kernels and
never calls them.

What it follows: Terminal Velocity Matching trains a DiT (Sec. "Experiments"; the layer equations of App. "Full
Description of Normalization of Modulation" call the block's second branch MLP and say nothing more about it), and
the network's JVP runs through that branch too (Sec. 4).  The MLP is taken to be DiT's: two linear layers around
the GELU in its tanh form,

    gelu(u) = u/2 (1 + tanh(k (u + c u^3))),   k = sqrt(2/pi),  c = 0.044715

(this reading is the repository's; the paper does not name the activation).  The linear layers are plain matrix
products and carry a tangent like any input; what is specific is the activation between them:

    a = gelu(u),   ta = gelu'(u) tu,

and the gradient of <ga, a> + <gta, ta> with respect to u and tu, which needs gelu''.  Derivatives are taken node by
node through  v = u + c u^3,  w = k v,  t = tanh(w),  a = u (1 + t) / 2  (forward mode for the tangent, then a
reverse sweep over the same nodes and their tangents), not from a collected closed form.

Pins (tests/test_gelu_oracle.py): torch's gelu(approximate="tanh") with torch.func.jvp and autograd in float64,
central finite differences for the tangent and both gradients, values at 0, the limits for large |u|, the identity
gelu(u) - gelu(-u) = u, linearity in the tangent.
"""
import numpy as np

K = np.sqrt(2.0 / np.pi)
C = 0.044715


def gelu_jvp_fwd(u, tu):
    """Returns (a, ta), same shape as u."""
    u, tu = np.asarray(u, dtype=np.float64), np.asarray(tu, dtype=np.float64)
    v = u + C * u ** 3
    tv = tu + 3.0 * C * u ** 2 * tu
    w, tw = K * v, K * tv
    t = np.tanh(w)
    tt = (1.0 - t * t) * tw
    a = 0.5 * u * (1.0 + t)
    ta = 0.5 * tu * (1.0 + t) + 0.5 * u * tt
    return a, ta


def gelu_jvp_bwd(u, tu, ga, gta):
    """Gradient of <ga, a> + <gta, ta> with respect to u and tu.  Returns (gu, gtu)."""
    u, tu, ga, gta = (np.asarray(x, dtype=np.float64) for x in (u, tu, ga, gta))
    # forward nodes again
    tv = tu + 3.0 * C * u ** 2 * tu
    w, tw = K * (u + C * u ** 3), K * tv
    t = np.tanh(w)
    s = 1.0 - t * t
    tt = s * tw
    # reverse sweep: a = u (1 + t) / 2;  ta = tu (1 + t) / 2 + u tt / 2
    gu = 0.5 * ga * (1.0 + t) + 0.5 * gta * tt
    gtu = 0.5 * gta * (1.0 + t)
    g_t = 0.5 * ga * u + 0.5 * gta * tu
    g_tt = 0.5 * gta * u
    # tt = (1 - t^2) tw
    g_t = g_t - 2.0 * t * tw * g_tt
    g_tw = s * g_tt
    # t = tanh(w)
    g_w = s * g_t
    # w = K v, tw = K tv
    g_v, g_tv = K * g_w, K * g_tw
    # v = u + C u^3;  tv = tu + 3 C u^2 tu
    gu = gu + g_v * (1.0 + 3.0 * C * u ** 2) + g_tv * 6.0 * C * u * tu
    gtu = gtu + g_tv * (1.0 + 3.0 * C * u ** 2)
    return gu, gtu
