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


def elem_err(got, ref):
    """The elementwise companion of rel_err, reported beside it: max over the elements of
    |gpu - ref| / (|ref| + rms(ref)), which does not let one large entry hide errors in the small ones."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    if rms < 1e-6:
        rms = 1.0
    return float((np.abs(got - ref) / (np.abs(ref) + rms)).max())


def run_gpu(inp, scale=0.0, flags=0):
    """inp: dict of CPU tensors (workloads.make_inputs).  Returns (fwd tuple, bwd tuple) on the GPU."""
    dev = {n: t.cuda() for n, t in inp.items()}
    o, to, lse, stats = tvm.tvmattn_jvp_fwd(dev["q"], dev["k"], dev["v"], dev["tq"], dev["tk"], dev["tv"], scale,
                                            flags=flags)
    grads = tvm.tvmattn_jvp_bwd(dev["q"], dev["k"], dev["v"], dev["tq"], dev["tk"], dev["tv"], o, to, lse, stats,
                                dev["gO"], dev["gTO"], scale, flags=flags)
    torch.cuda.synchronize()
    return (o, to, lse, stats), grads


def check_heads(w, inp, fwd, grads, heads, scale=None, tol=None, report=None):
    """Element-by-element comparison with the oracle on the listed (b,h) heads.  Asserts the per-tensor
    max |gpu - ref| / max |ref| bound; returns those worst values and, in `report` (a dict, if given), the worst
    elementwise |gpu - ref| / (|ref| + rms(ref)) per tensor as well."""
    tol = TOL[w.dtype] if tol is None else tol
    worst, worst_elem = {}, {}
    # one device-to-host copy per tensor (float32 holds bf16 and float32 results exactly)
    got_host = [t.float().cpu().numpy() for t in list(fwd) + list(grads)]
    for (b, h) in heads:
        a = [wl.to_f64(inp[n][b, h]) for n in wl.NAMES]
        ro = orc.attn_jvp_fwd_head(*a[:6], scale)
        rg = orc.attn_jvp_bwd_head(*a, scale)
        for name, got, ref in zip(FWD_NAMES + BWD_NAMES, got_host, list(ro) + list(rg)):
            worst[name] = max(worst.get(name, 0.0), rel_err(got[b, h], ref))
            worst_elem[name] = max(worst_elem.get(name, 0.0), elem_err(got[b, h], ref))
    print("   max|err|/max|ref|      :", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)
    print("   max |err|/(|ref|+rms)  :", {k: f"{v:.2e}" for k, v in worst_elem.items()}, flush=True)
    if report is not None:
        report.update(worst_elem)
    bad = {k: v for k, v in worst.items() if not (v <= tol)}
    assert not bad, f"{w.name}: rel err above {tol}: {bad} (all: {worst})"
    return worst


def all_heads(w):
    return [(b, h) for b in range(w.B) for h in range(w.H)]
