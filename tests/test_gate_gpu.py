"""GPU-vs-oracle parity of the normalised residual-gate entry points through the C-ABI.  Every case prints its
name before touching the GPU."""
import sys

import numpy as np
import pytest
import torch

import paper_2511_19797_amd as tvm
from oracle import gate_oracle as orc
from paper_2511_19797_amd import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
EPS = 1e-6


def announce(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def run(inp):
    dev = {n: t.cuda() for n, t in inp.items()}
    z, tz = tvm.tvmattn_gate_jvp_fwd(dev["x"], dev["tx"], dev["h"], dev["th"], dev["c"], dev["tc"], EPS)
    grads = tvm.tvmattn_gate_jvp_bwd(dev["h"], dev["th"], dev["c"], dev["tc"], EPS, dev["gz"], dev["gtz"])
    torch.cuda.synchronize()
    return (z, tz), grads


NAMES = ("z", "tz", "gh", "gth", "gc", "gtc")


def check(inp, fwd, grads, dtype):
    f = {n: wl.to_f64(t) for n, t in inp.items()}
    six = [f[n] for n in ("x", "tx", "h", "th", "c", "tc")]
    ref = list(orc.gate_jvp_fwd(*six, EPS)) + list(orc.gate_jvp_bwd(*six, EPS, f["gz"], f["gtz"])[2:])
    worst = {n: pu.rel_err(g.float().cpu().numpy(), r) for n, g, r in zip(NAMES, list(fwd) + list(grads), ref)}
    bad = {k: v for k, v in worst.items() if not (v <= pu.TOL[dtype])}
    assert not bad, f"rel err above {pu.TOL[dtype]}: {bad} (all: {worst})"
    return worst


@pytest.mark.parametrize("B,T,C,dtype", [
    (1, 1, 8, "bf16"), (2, 7, 64, "bf16"), (3, 50, 512, "bf16"), (2, 130, 768, "bf16"), (2, 65, 1152, "bf16"),
    (1, 9, 1536, "bf16"), (1, 5, 2048, "bf16"), (2, 33, 4, "f32"), (2, 21, 260, "f32"), (1, 6, 1024, "f32"),
    (70, 3, 128, "bf16"), (300, 23, 64, "bf16"),   # the last: several passes per workgroup and a ragged last one
])
def test_every_element_against_the_oracle(B, T, C, dtype):
    announce(f"gate B{B} T{T} C{C} {dtype}")
    inp = wl.make_gate_inputs(B, T, C, dtype, 91)
    fwd, grads = run(inp)
    worst = check(inp, fwd, grads, dtype)
    print("   worst rel err:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)


def test_full_size_and_reproducible():
    """DiT-XL/2 at 512 px: 16 images x 1024 tokens x 1152 features (the shape bench.py times): every element, and
    two runs agree bit for bit."""
    announce("gate full size B16 T1024 C1152 bf16")
    inp = wl.make_gate_inputs(16, 1024, 1152, "bf16", 92)
    fwd, grads = run(inp)
    check(inp, fwd, grads, "bf16")
    fwd2, grads2 = run(inp)
    for a, b in zip(list(fwd) + list(grads), list(fwd2) + list(grads2)):
        assert torch.equal(a, b)


def test_open_gate_is_a_plain_residual_add():
    """A constant gate normalises to ones (up to eps): z = x + h and tz = tx + th, and with float32 exactly so
    up to the rounding of 1/sqrt(1 + eps)."""
    announce("gate constant c, f32")
    inp = wl.make_gate_inputs(2, 9, 64, "f32", 93)
    inp["c"] = torch.full_like(inp["c"], 2.5)
    inp["tc"] = torch.zeros_like(inp["tc"])
    dev = {n: t.cuda() for n, t in inp.items()}
    z, tz = tvm.tvmattn_gate_jvp_fwd(dev["x"], dev["tx"], dev["h"], dev["th"], dev["c"], dev["tc"], EPS)
    torch.cuda.synchronize()
    assert torch.allclose(z.cpu(), inp["x"] + inp["h"], rtol=1e-5, atol=1e-5)
    assert torch.allclose(tz.cpu(), inp["tx"] + inp["th"], rtol=1e-5, atol=1e-5)


def test_unsupported_sizes_raise():
    announce("gate unsupported sizes")
    inp = wl.make_gate_inputs(1, 2, 2056, "bf16", 94)   # more than 256 chunks of 8
    dev = {n: t.cuda() for n, t in inp.items()}
    with pytest.raises(tvm.TvmattnError):
        tvm.tvmattn_gate_jvp_fwd(dev["x"], dev["tx"], dev["h"], dev["th"], dev["c"], dev["tc"], EPS)
    with pytest.raises(tvm.TvmattnError):
        tvm.tvmattn_gate_jvp_bwd(dev["h"], dev["th"], dev["c"], dev["tc"], EPS, dev["gz"], dev["gtz"])


def test_stream_updated_in_place():
    """z = x and tz = tx as the same buffers: the same bits as the out-of-place call."""
    announce("gate in place B2 T130 C1152 bf16")
    inp = wl.make_gate_inputs(2, 130, 1152, "bf16", 95)
    dev = {n: t.cuda() for n, t in inp.items()}
    z, tz = tvm.tvmattn_gate_jvp_fwd(dev["x"], dev["tx"], dev["h"], dev["th"], dev["c"], dev["tc"], EPS)
    x, tx = dev["x"].clone(), dev["tx"].clone()
    tvm.tvmattn_gate_jvp_fwd(x, tx, dev["h"], dev["th"], dev["c"], dev["tc"], EPS, out=(x, tx))
    torch.cuda.synchronize()
    assert torch.equal(x, z) and torch.equal(tx, tz)
    with pytest.raises(tvm.TvmattnError):   # any other aliasing is refused
        tvm.tvmattn_gate_jvp_fwd(dev["x"], dev["tx"], dev["h"], dev["th"], dev["c"], dev["tc"], EPS, out=(dev["tx"], tz))
