"""The linear layer with tangent and its backward on the GPU (through the C-ABI) against the float64 oracle,
element by element."""
import sys

import numpy as np
import pytest
import torch

import paper_2511_19797_amd as tvm
from oracle import linear_oracle as orc
from paper_2511_19797_amd import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
TOL = 2e-2   # bf16 storage, float32 accumulation: max |gpu - ref| / max |ref| per tensor
NAMES = ("y", "ty", "gx", "gtx", "gw", "gb")


def run(R, K, F, seed, bias=True):
    print(f"[case] linear R={R} K={K} F={F} bias={bias} seed={seed}", flush=True)
    sys.stdout.flush()
    inp = wl.make_linear_inputs(R, K, F, "bf16", seed)
    d = {n: t.cuda() for n, t in inp.items()}
    y, ty = tvm.tvmattn_linear_jvp_fwd(d["x"], d["tx"], d["w"], d["b"] if bias else None)
    gx, gtx, gw, gb = tvm.tvmattn_linear_jvp_bwd(d["x"], d["tx"], d["w"], d["gy"], d["gty"], bias_grad=bias)
    torch.cuda.synchronize()
    f = {n: wl.to_f64(t) for n, t in inp.items()}
    ry, rty = orc.linear_jvp_fwd(f["x"], f["tx"], f["w"], f["b"] if bias else None)
    rgx, rgtx, rgw, rgb = orc.linear_jvp_bwd(f["x"], f["tx"], f["w"], f["gy"], f["gty"])
    got = [y, ty, gx, gtx, gw] + ([gb] if bias else [])
    ref = [ry, rty, rgx, rgtx, rgw] + ([rgb] if bias else [])
    worst, elem = {}, {}
    for name, g, r in zip(NAMES, got, ref):
        g = g.float().cpu().numpy()
        worst[name], elem[name] = pu.rel_err(g, r), pu.elem_err(g, r)
    print("   max|err|/max|ref|      :", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)
    print("   max |err|/(|ref|+rms)  :", {k: f"{v:.2e}" for k, v in elem.items()}, flush=True)
    bad = {k: v for k, v in worst.items() if not (v <= TOL)}
    assert not bad, bad
    if not bias:
        assert gb is None


@pytest.mark.parametrize("R,K,F", [
    (1, 32, 32),          # one token, one block of everything
    (31, 32, 64), (33, 64, 32),
    (100, 64, 96),        # ragged token count: a partial last contraction tile in the weight gradient
    (128, 256, 256),      # exactly one output tile
    (129, 96, 288),       # one row more than a tile; F beyond one column tile
    (257, 160, 544),      # three row tiles, ragged in every dimension of the tiling
    (300, 1152, 384), (300, 384, 1152),
    (1000, 288, 864),     # the shape of a QKV projection (F = 3 K) with many contraction splits
    (513, 64, 256),       # one row beyond two row tiles of 256; contraction of exactly one tile
    (600, 352, 608),      # contraction lengths that end in half a tile (352 = 5.5 x 64, 608 = 9.5 x 64)
    (4000, 1152, 3392),   # two rounds of persistent workgroups, ragged in rows and columns
])
def test_linear_against_the_oracle(R, K, F):
    run(R, K, F, seed=7 + R % 5)


def test_linear_without_bias_and_bitwise_reproducible():
    run(200, 128, 192, seed=3, bias=False)
    inp = wl.make_linear_inputs(333, 192, 320, "bf16", 4)
    d = {n: t.cuda() for n, t in inp.items()}
    a = tvm.tvmattn_linear_jvp_bwd(d["x"], d["tx"], d["w"], d["gy"], d["gty"])
    b = tvm.tvmattn_linear_jvp_bwd(d["x"], d["tx"], d["w"], d["gy"], d["gty"])
    torch.cuda.synchronize()
    for u, v in zip(a, b):
        assert torch.equal(u, v)


def test_linear_batched_shapes_and_the_tangent_is_the_forward_of_the_tangent():
    """[B,T,K] inputs; with no bias, ty is bit for bit the y of a call whose x is tx (the two row sets run the same code)."""
    inp = wl.make_linear_inputs(2 * 77, 96, 160, "bf16", 5)
    x, tx, w = (inp[n].cuda() for n in ("x", "tx", "w"))
    x3, tx3 = x.view(2, 77, 96), tx.view(2, 77, 96)
    y, ty = tvm.tvmattn_linear_jvp_fwd(x3, tx3, w)
    y2, _ = tvm.tvmattn_linear_jvp_fwd(tx3, x3, w)
    torch.cuda.synchronize()
    assert y.shape == (2, 77, 160) and torch.equal(ty, y2)


def test_linear_on_slices_of_wider_buffers():
    """x and tx as slices of one [R, 3K] buffer (how an attention output laid out like its fused-projection queries
    reaches the output projection), y and ty written into slices of a [R, 2F + 64] buffer, and the same layouts for the
    backward's gradients: against the oracle, and bit for bit against the call on dense copies."""
    R, K, F = 300, 96, 160
    inp = wl.make_linear_inputs(R, K, F, "bf16", 21)
    d = {n: t.cuda() for n, t in inp.items()}
    xb = torch.zeros(R, 3 * K, dtype=torch.bfloat16, device="cuda")
    xb[:, :K], xb[:, 2 * K:] = d["x"], d["tx"]
    xs, txs = xb[:, :K], xb[:, 2 * K:]
    yb = torch.full((R, 2 * F + 64), float("nan"), dtype=torch.bfloat16, device="cuda")
    ys, tys = yb[:, :F], yb[:, F + 64:]
    tvm.tvmattn_linear_jvp_fwd(xs, txs, d["w"], d["b"], out=(ys, tys))
    y, ty = tvm.tvmattn_linear_jvp_fwd(d["x"], d["tx"], d["w"], d["b"])
    gb_ = torch.zeros(R, 2 * F + 64, dtype=torch.bfloat16, device="cuda")
    gb_[:, :F], gb_[:, F + 64:] = d["gy"], d["gty"]
    gxb = torch.full((R, 3 * K), float("nan"), dtype=torch.bfloat16, device="cuda")
    out = (gxb[:, :K], gxb[:, 2 * K:], torch.empty_like(d["w"]), torch.empty(F, dtype=torch.bfloat16, device="cuda"))
    tvm.tvmattn_linear_jvp_bwd(xs, txs, d["w"], gb_[:, :F], gb_[:, F + 64:], out=out)
    ref = tvm.tvmattn_linear_jvp_bwd(d["x"], d["tx"], d["w"], d["gy"], d["gty"])
    torch.cuda.synchronize()
    assert torch.equal(ys, y) and torch.equal(tys, ty)
    for a, b in zip(out, ref):
        assert torch.equal(a, b)
    assert bool(torch.isnan(yb[:, F:F + 64].float()).all()) and bool(torch.isnan(gxb[:, K:2 * K].float()).all())  # gaps untouched
    f = {n: wl.to_f64(t) for n, t in inp.items()}
    assert pu.rel_err(ys.float().cpu().numpy(), orc.linear_jvp_fwd(f["x"], f["tx"], f["w"], f["b"])[0]) <= TOL


@pytest.mark.parametrize("K,F", [(1152, 1152), (1152, 4608), (4608, 1152), (1152, 3456)])
def test_linear_at_the_block_sizes(K, F):
    """The layers of a DiT-XL/2 block at 512 px (16 x 1024 tokens; hidden 1152, MLP width 4608, fused QKV 3456), at the
    size bench.py times, a quarter of the tokens for the oracle's sake on the widest ones."""
    run(16 * 1024 if K * F <= 1152 * 1152 else 4 * 1024, K, F, seed=11)


def test_unsupported_shapes_are_refused():
    x = torch.zeros(10, 40, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(64, 40, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(tvm.TvmattnError) as e:
        tvm.tvmattn_linear_jvp_fwd(x, x.clone(), w)
    assert e.value.status == -2
    xf = torch.zeros(10, 64, dtype=torch.float32, device="cuda")
    wf = torch.zeros(64, 64, dtype=torch.float32, device="cuda")
    with pytest.raises(tvm.TvmattnError) as e:
        tvm.tvmattn_linear_jvp_fwd(xf, xf.clone(), wf)
    assert e.value.status == -2
