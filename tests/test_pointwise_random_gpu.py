"""Sixteen seeded random problems (shapes, dtypes, eps, scales of the pre-activations, with and without the residual
gradients) for the pointwise entry points against their oracles, every element.  Each case prints its name before
touching the GPU."""
import random

import pytest
import torch

import paper_2511_19797_amd as tvm
from oracle import adaln_oracle as ao
from oracle import gate_oracle as go
from oracle import gelu_oracle as eo
from paper_2511_19797_amd import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def test_random_problems_against_the_oracles():
    rnd = random.Random(5)
    worst = 0.0
    for it in range(16):
        dtype = rnd.choice(["bf16", "bf16", "f32"])
        vec = 8 if dtype == "bf16" else 4
        C = vec * rnd.randint(1, 256)
        B = rnd.choice([1, 1, 2, 3, 5, 17])
        T = rnd.choice([1, 2, 3, 5, 8, 31, 64, 100, 257])
        if B * T * C > 3_000_000: T = max(1, 3_000_000 // (B * C))
        eps = rnd.choice([0.0, 1e-6, 1e-3])
        print(f"[case {it}] B{B} T{T} C{C} {dtype} eps{eps}", flush=True)
        tol = pu.TOL[dtype]
        a = wl.make_adaln_inputs(B, T, C, dtype, 1000 + it); d = {n: t.cuda() for n, t in a.items()}
        six = [d[n] for n in ("x", "tx", "a", "ta", "b", "tb")]
        res = wl.make_gate_inputs(B, T, C, dtype, 3000 + it)
        use_res = it % 2 == 0
        got = list(tvm.tvmattn_adaln_jvp_fwd(*six, eps)) + list(tvm.tvmattn_adaln_jvp_bwd(*six, eps, d["gy"], d["gty"], gres=res["gz"].cuda() if use_res else None, gtres=res["gtz"].cuda() if use_res else None))
        torch.cuda.synchronize()
        f = {n: wl.to_f64(t) for n, t in a.items()}
        s6 = [f[n] for n in ("x", "tx", "a", "ta", "b", "tb")]
        ref = list(ao.adaln_jvp_fwd(*s6, eps)) + list(ao.adaln_jvp_bwd(*s6, eps, f["gy"], f["gty"]))
        if use_res:
            ref[2] = ref[2] + wl.to_f64(res["gz"]); ref[3] = ref[3] + wl.to_f64(res["gtz"])
        for k, (g, r) in enumerate(zip(got, ref)):
            e = pu.rel_err(g.float().cpu().numpy(), r); worst = max(worst, e / tol)
            assert e <= tol, ("adaln", k, e)
        g_ = {n: t.cuda() for n, t in res.items()}
        got = list(tvm.tvmattn_gate_jvp_fwd(g_["x"], g_["tx"], g_["h"], g_["th"], g_["c"], g_["tc"], eps)) + list(tvm.tvmattn_gate_jvp_bwd(g_["h"], g_["th"], g_["c"], g_["tc"], eps, g_["gz"], g_["gtz"]))
        torch.cuda.synchronize()
        f = {n: wl.to_f64(t) for n, t in res.items()}
        s6 = [f[n] for n in ("x", "tx", "h", "th", "c", "tc")]
        ref = list(go.gate_jvp_fwd(*s6, eps)) + list(go.gate_jvp_bwd(*s6, eps, f["gz"], f["gtz"])[2:])
        for k, (g, r) in enumerate(zip(got, ref)):
            e = pu.rel_err(g.float().cpu().numpy(), r); worst = max(worst, e / tol)
            assert e <= tol, ("gate", k, e)
        e_ = wl.make_gelu_inputs((B, T, C), dtype, 5000 + it); de = {n: (t * rnd.choice([0.1, 1.0, 4.0])).contiguous() for n, t in e_.items()}
        dd = {n: t.cuda() for n, t in de.items()}
        got = list(tvm.tvmattn_gelu_jvp_fwd(dd["u"], dd["tu"])) + list(tvm.tvmattn_gelu_jvp_bwd(dd["u"], dd["tu"], dd["ga"], dd["gta"]))
        torch.cuda.synchronize()
        f = {n: wl.to_f64(t) for n, t in de.items()}
        ref = list(eo.gelu_jvp_fwd(f["u"], f["tu"])) + list(eo.gelu_jvp_bwd(f["u"], f["tu"], f["ga"], f["gta"]))
        for k, (g, r) in enumerate(zip(got, ref)):
            e = pu.rel_err(g.float().cpu().numpy(), r); worst = max(worst, e / tol)
            assert e <= tol, ("gelu", k, e)
    print("worst error / tolerance:", worst, flush=True)
