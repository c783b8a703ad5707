"""GPU-vs-oracle parity of the MLP activation (tanh-form GELU with tangent and backward) through the C-ABI.  Every
case prints its name before touching the GPU."""
import sys

import numpy as np
import pytest
import torch

import paper_2511_19797_amd as tvm
from oracle import gelu_oracle as orc
from paper_2511_19797_amd import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
NAMES = ("a", "ta", "gu", "gtu")


def announce(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def run(inp):
    dev = {n: t.cuda() for n, t in inp.items()}
    fwd = tvm.tvmattn_gelu_jvp_fwd(dev["u"], dev["tu"])
    bwd = tvm.tvmattn_gelu_jvp_bwd(dev["u"], dev["tu"], dev["ga"], dev["gta"])
    torch.cuda.synchronize()
    return list(fwd) + list(bwd)


def check(inp, got, dtype):
    f = {n: wl.to_f64(t) for n, t in inp.items()}
    ref = list(orc.gelu_jvp_fwd(f["u"], f["tu"])) + list(orc.gelu_jvp_bwd(f["u"], f["tu"], f["ga"], f["gta"]))
    worst = {n: pu.rel_err(g.float().cpu().numpy(), r) for n, g, r in zip(NAMES, got, ref)}
    bad = {k: v for k, v in worst.items() if not (v <= pu.TOL[dtype])}
    assert not bad, f"rel err above {pu.TOL[dtype]}: {bad} (all: {worst})"
    return worst


@pytest.mark.parametrize("shape,dtype", [
    ((8,), "bf16"), ((4,), "f32"), ((3, 40), "bf16"), ((1000, 8), "bf16"), ((257, 1024), "bf16"), ((7, 13, 64), "f32"),
    ((2, 130, 4608), "bf16"), ((1048584,), "f32"),   # the last two: several chunks per thread and a ragged last turn
])
def test_every_element_against_the_oracle(shape, dtype):
    announce(f"gelu {shape} {dtype}")
    inp = wl.make_gelu_inputs(shape, dtype, 101)
    worst = check(inp, run(inp), dtype)
    print("   worst rel err:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)


def test_wide_range_of_pre_activations():
    """Large |u| (tanh saturated, exp overflowing to inf or underflowing to 0) and tiny ones stay finite and right."""
    announce("gelu wide range f32")
    u = torch.tensor([0.0, 1e-6, -1e-6, 0.5, -0.5, 3.0, -3.0, 9.0, -9.0, 40.0, -40.0, 300.0, -300.0, 1e4, -1e4, 2.0],
                     dtype=torch.float32)
    inp = {"u": u, "tu": torch.ones_like(u), "ga": torch.ones_like(u), "gta": torch.full_like(u, 0.5)}
    got = run(inp)
    f = {n: wl.to_f64(t) for n, t in inp.items()}
    ref = list(orc.gelu_jvp_fwd(f["u"], f["tu"])) + list(orc.gelu_jvp_bwd(f["u"], f["tu"], f["ga"], f["gta"]))
    for n, g, r in zip(NAMES, got, ref):
        g = g.cpu().numpy().astype(np.float64)
        assert np.isfinite(g).all(), n
        assert np.allclose(g, r, rtol=2e-5, atol=2e-6), (n, g, r)


def test_full_size_and_reproducible():
    """The hidden layer of DiT-XL/2's MLP at 512 px: 16 x 1024 tokens x 4608 features (the shape bench.py times),
    sampled rows against the oracle, two runs bit for bit."""
    announce("gelu full size 16x1024x4608 bf16")
    inp = wl.make_gelu_inputs((16, 1024, 4608), "bf16", 102)
    got = run(inp)
    again = run(inp)
    for a, b in zip(got, again):
        assert torch.equal(a, b)
    rows = [(0, 0), (3, 511), (15, 1023), (8, 77)]
    sub = {n: torch.stack([t[b, r] for b, r in rows]) for n, t in inp.items()}
    check(sub, [torch.stack([g[b, r] for b, r in rows]) for g in got], "bf16")


def test_unsupported_sizes_raise():
    announce("gelu unsupported sizes")
    inp = wl.make_gelu_inputs((12,), "bf16", 103)
    dev = {n: t.cuda() for n, t in inp.items()}
    with pytest.raises(tvm.TvmattnError):
        tvm.tvmattn_gelu_jvp_fwd(dev["u"], dev["tu"])
