"""GPU-vs-oracle parity of the normalised AdaLN modulation entry points through the C-ABI.  Every case prints
its name before touching the GPU."""
import sys

import numpy as np
import pytest
import torch

import paper_2511_19797_amd as tvm
from oracle import adaln_oracle as orc
from paper_2511_19797_amd import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
EPS = 1e-6


def announce(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def run(inp):
    dev = {n: t.cuda() for n, t in inp.items()}
    y, ty = tvm.tvmattn_adaln_jvp_fwd(dev["x"], dev["tx"], dev["a"], dev["ta"], dev["b"], dev["tb"], EPS)
    grads = tvm.tvmattn_adaln_jvp_bwd(dev["x"], dev["tx"], dev["a"], dev["ta"], dev["b"], dev["tb"], EPS, dev["gy"],
                                      dev["gty"])
    torch.cuda.synchronize()
    return (y, ty), grads


NAMES = ("y", "ty", "gx", "gtx", "ga", "gta", "gb", "gtb")


def check(inp, fwd, grads, dtype):
    f = {n: wl.to_f64(t) for n, t in inp.items()}
    ref = list(orc.adaln_jvp_fwd(f["x"], f["tx"], f["a"], f["ta"], f["b"], f["tb"], EPS))
    ref += list(orc.adaln_jvp_bwd(f["x"], f["tx"], f["a"], f["ta"], f["b"], f["tb"], EPS, f["gy"], f["gty"]))
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
    announce(f"adaln B{B} T{T} C{C} {dtype}")
    inp = wl.make_adaln_inputs(B, T, C, dtype, 81)
    fwd, grads = run(inp)
    worst = check(inp, fwd, grads, dtype)
    print("   worst rel err:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)


def test_full_size_and_reproducible():
    """DiT-XL/2 at 512 px: 16 images x 1024 tokens x 1152 features (the shape bench.py times): every element, and
    two runs agree bit for bit."""
    announce("adaln full size B16 T1024 C1152 bf16")
    inp = wl.make_adaln_inputs(16, 1024, 1152, "bf16", 82)
    fwd, grads = run(inp)
    check(inp, fwd, grads, "bf16")
    fwd2, grads2 = run(inp)
    for p, q in zip(list(fwd) + list(grads), list(fwd2) + list(grads2)):
        assert torch.equal(p, q)


def test_unsupported_sizes_are_refused():
    announce("adaln unsupported sizes")
    inp = wl.make_adaln_inputs(1, 2, 2056, "bf16", 83)   # more than 256 chunks of 8
    dev = {n: t.cuda() for n, t in inp.items()}
    with pytest.raises(tvm.TvmattnError) as ei:
        tvm.tvmattn_adaln_jvp_fwd(dev["x"], dev["tx"], dev["a"], dev["ta"], dev["b"], dev["tb"], EPS)
    assert ei.value.status == -2
    inp = wl.make_adaln_inputs(1, 2, 12, "bf16", 84)     # not a whole number of 16-byte chunks
    dev = {n: t.cuda() for n, t in inp.items()}
    with pytest.raises(tvm.TvmattnError) as ei:
        tvm.tvmattn_adaln_jvp_fwd(dev["x"], dev["tx"], dev["a"], dev["ta"], dev["b"], dev["tb"], EPS)
    assert ei.value.status == -2


def test_backward_with_the_residual_gradients_added():
    """gres, gtres are added to gx, gtx: the gradient of <gy,y> + <gty,ty> + <gres,x> + <gtres,tx>.  The other four
    gradients are those of the plain call, bit for bit."""
    for B, T, C, dtype in ((2, 37, 1152, "bf16"), (1, 9, 260, "f32")):
        announce(f"adaln backward with residual gradients B{B} T{T} C{C} {dtype}")
        inp = wl.make_adaln_inputs(B, T, C, dtype, 85)
        res = wl.make_gate_inputs(B, T, C, dtype, 86)      # any two [B,T,C] tensors: its gz, gtz
        dev = {n: t.cuda() for n, t in inp.items()}
        gres, gtres = res["gz"].cuda(), res["gtz"].cuda()
        six = [dev[n] for n in ("x", "tx", "a", "ta", "b", "tb")]
        plain = tvm.tvmattn_adaln_jvp_bwd(*six, EPS, dev["gy"], dev["gty"])
        fused = tvm.tvmattn_adaln_jvp_bwd(*six, EPS, dev["gy"], dev["gty"], gres=gres, gtres=gtres)
        torch.cuda.synchronize()
        for k in range(2, 6):
            assert torch.equal(plain[k], fused[k])
        f = {n: wl.to_f64(t) for n, t in inp.items()}
        ref = orc.adaln_jvp_bwd(f["x"], f["tx"], f["a"], f["ta"], f["b"], f["tb"], EPS, f["gy"], f["gty"])
        want = (ref[0] + wl.to_f64(res["gz"]), ref[1] + wl.to_f64(res["gtz"]))
        for k in range(2):
            e = pu.rel_err(fused[k].float().cpu().numpy(), want[k])
            assert e <= pu.TOL[dtype], (k, e)
        with pytest.raises(ValueError):
            tvm.tvmattn_adaln_jvp_bwd(*six, EPS, dev["gy"], dev["gty"], gres=gres)
