"""One normalised DiT block with tangent, forward and backward, as a chain of the library's entry points on the GPU
(every stage consumes the bf16 outputs of the stage before it) against the chained float64 oracles on the same stored
inputs and weights: the block's two outputs and every gradient (stream, tangent, twelve modulation tensors, all
weights, biases and gains)."""
import sys

import numpy as np
import pytest
import torch

from oracle import block_oracle as orc
from paper_2511_19797_amd import block, workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
EPS, QK_EPS = 1e-6, 1e-6
# Every stage rounds its outputs to bf16 (2^-9 relative per element) and the stages' own bound is 2e-2; a chain of
# ten stages accumulates independent roundings: measured worst 1.7e-2 (the QK-norm gains' gradients, sums over every
# row of every head of the batch), 4e-3 to 8e-3 for the other tensors.
TOL = 4e-2


@pytest.mark.parametrize("B,T,H,d,hidden", [
    (2, 200, 4, 72, 1152),     # padded head dim, ragged token count, the fused norm backward
    (1, 130, 2, 64, 256),
    (1, 96, 1, 128, 512),      # head dim beyond the fused norm backward: attention backward and norm backward as two calls
    (1, 256, 16, 72, 4608),    # DiT-XL/2 width at 256 px, one batch element
])
def test_block_chain_against_the_chained_oracles(B, T, H, d, hidden):
    print(f"[case] block B={B} T={T} H={H} d={d} hidden={hidden}", flush=True)
    sys.stdout.flush()
    x, tx, mods, tmods, params, gz, gtz = wl.make_block_inputs(B, T, H, d, hidden, seed=17 + T)
    dev = lambda t: t.cuda()
    dm, dtm, dp = ({k: dev(v) for k, v in m.items()} for m in (mods, tmods, params))
    z, tz, saved = block.block_jvp_fwd(dev(x), dev(tx), dm, dtm, dp, H, EPS, QK_EPS)
    g = block.block_jvp_bwd(dev(x), dev(tx), dm, dtm, dp, H, EPS, QK_EPS, saved, dev(gz), dev(gtz))
    torch.cuda.synchronize()
    f = wl.to_f64
    fm, ftm, fp = ({k: f(v) for k, v in m.items()} for m in (mods, tmods, params))
    rz, rtz = orc.block_jvp_fwd(f(x), f(tx), fm, ftm, fp, H, EPS, QK_EPS)
    rg = orc.block_jvp_bwd(f(x), f(tx), fm, ftm, fp, H, EPS, QK_EPS, f(gz), f(gtz))
    worst, elem = {}, {}
    pairs = [("z", z, rz), ("tz", tz, rtz)] + [(k, g[k], rg[k]) for k in rg]
    assert set(g) == set(rg)
    for name, got, ref in pairs:
        got = got.float().cpu().numpy()
        worst[name], elem[name] = pu.rel_err(got.reshape(ref.shape), ref), pu.elem_err(got.reshape(ref.shape), ref)
    print("   max|err|/max|ref|      :", {k: f"{v:.1e}" for k, v in worst.items()}, flush=True)
    print("   max |err|/(|ref|+rms)  :", {k: f"{v:.1e}" for k, v in elem.items()}, flush=True)
    bad = {k: v for k, v in worst.items() if not (v <= TOL)}
    assert not bad, bad
