"""Helpers shared by the GPU parity tests: run the library, run the oracle, compare."""
import numpy as np
import torch

import paper_2511_19797_amd as tvm
from oracle import tvmattn_oracle as orc
from paper_2511_19797_amd import workloads as wl

# max |gpu - ref| / max |ref| per output tensor (the benchmark spec's tolerances).
TOL = {"f32": 1e-4, "bf16": 2e-2}

FWD_NAMES = ("o", "to", "lse", "stats")
BWD_NAMES = ("dq", "dk", "dv", "dtq", "dtk", "dtv")


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite values in GPU result"
    denom = float(np.abs(ref).max())
    if denom < 1e-6:
        # the reference is identically zero up to float64 rounding (single-token gradients, zero
        # tangents): inputs are O(1), so the error is taken absolutely
        denom = 1.0
    return float(np.abs(got - ref).max() / denom)


def run_gpu(inp, scale=0.0):
    """inp: dict of CPU tensors (workloads.make_inputs).  Returns (fwd tuple, bwd tuple) on the GPU."""
    dev = {n: t.cuda() for n, t in inp.items()}
    o, to, lse, stats = tvm.tvmattn_jvp_fwd(dev["q"], dev["k"], dev["v"], dev["tq"], dev["tk"], dev["tv"], scale)
    grads = tvm.tvmattn_jvp_bwd(dev["q"], dev["k"], dev["v"], dev["tq"], dev["tk"], dev["tv"], o, to, lse, stats,
                                dev["gO"], dev["gTO"], scale)
    torch.cuda.synchronize()
    return (o, to, lse, stats), grads


def check_heads(w, inp, fwd, grads, heads, scale=None, tol=None):
    """Element-by-element comparison with the oracle on the listed (b,h) heads."""
    tol = TOL[w.dtype] if tol is None else tol
    worst = {}
    for (b, h) in heads:
        a = [wl.to_f64(inp[n][b, h]) for n in wl.NAMES]
        ro = orc.attn_jvp_fwd_head(*a[:6], scale)
        rg = orc.attn_jvp_bwd_head(*a, scale)
        for name, got, ref in list(zip(FWD_NAMES, fwd, ro)) + list(zip(BWD_NAMES, grads, rg)):
            e = rel_err(got[b, h].float().cpu().numpy(), ref)
            worst[name] = max(worst.get(name, 0.0), e)
    bad = {k: v for k, v in worst.items() if not (v <= tol)}
    assert not bad, f"{w.name}: rel err above {tol}: {bad} (all: {worst})"
    return worst


def all_heads(w):
    return [(b, h) for b in range(w.B) for h in range(w.H)]
