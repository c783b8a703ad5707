"""The library under HIP graph capture: it allocates nothing, clears nothing with memsets and never synchronises,
so a forward + backward step captured once replays with the same bits as the eager calls.  Every replay is
checked, with eager work and synchronisations in between."""
import sys

import pytest
import torch

import paper_2511_19797_amd as tvm
from paper_2511_19797_amd import workloads as wl

pytestmark = pytest.mark.gpu


def announce(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("B,H,N,d,dtype", [(2, 4, 256, 72, "bf16"), (1, 2, 200, 64, "bf16"), (1, 2, 64, 32, "f32")])
def test_captured_step_replays_bit_for_bit(B, H, N, d, dtype):
    announce(f"graph capture B{B} H{H} N{N} d{d} {dtype}")
    w = wl.custom(B, H, N, d, dtype)
    dev = {n: t.cuda() for n, t in wl.make_inputs(w, 7).items()}
    six = [dev[n] for n in wl.NAMES[:6]]
    # eager reference
    fo = tvm.tvmattn_jvp_fwd(*six)
    go = tvm.tvmattn_jvp_bwd(*six, *fo, dev["gO"], dev["gTO"])
    torch.cuda.synchronize()
    ref = [t.clone() for t in list(fo) + list(go)]
    # buffers of the captured step: outputs and workspace allocated beforehand
    cf = tuple(torch.empty_like(t) for t in fo)
    cg = tuple(torch.empty_like(t) for t in go)
    ws = torch.empty(max(tvm.tvmattn_jvp_bwd_workspace_bytes(six[0]), 16), dtype=torch.uint8, device="cuda")

    def step():
        tvm.tvmattn_jvp_fwd(*six, out=cf)
        tvm.tvmattn_jvp_bwd(*six, *cf, dev["gO"], dev["gTO"], out=cg, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for replay in range(4):
        for t in cf + cg:  # eager work between the replays: the outputs are wiped with a fill kernel
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, want in zip(("o", "to", "lse", "stats", "dq", "dk", "dv", "dtq", "dtk", "dtv"), cf + cg, ref):
            assert torch.equal(got, want), f"replay {replay}: {name} differs from the eager call"


def test_captured_block_pieces_replay_bit_for_bit():
    """The entry points of the block (AdaLN modulation, QK-norm, the fused attention + QK-norm backward, gate,
    activation, a linear layer) in one captured graph, forward pieces and backward pieces."""
    announce("graph capture of the pointwise entry points")
    B, T, C, H, d, eps = 2, 130, 576, 8, 72, 1e-6
    a = {n: t.cuda() for n, t in wl.make_adaln_inputs(B, T, C, "bf16", 11).items()}
    g = {n: t.cuda() for n, t in wl.make_gate_inputs(B, T, C, "bf16", 12).items()}
    e = {n: t.cuda() for n, t in wl.make_gelu_inputs((B, T, 4 * C), "bf16", 13).items()}
    w = wl.custom(B, H, T, d, "bf16")
    q = {n: t.cuda() for n, t in wl.make_inputs(w, 14).items()}
    gq, gk = [t.cuda() for t in wl.make_gains(w, 15)]
    lin = {n: t.cuda() for n, t in wl.make_linear_inputs(B * T, C, 3 * C, "bf16", 16).items()}
    ws = torch.empty(max(1 << 24, tvm.tvmattn_linear_jvp_bwd_workspace_bytes(lin["x"], lin["w"])), dtype=torch.uint8, device="cuda")

    def calls(out):
        """out: None (eager, the binding allocates) or the list of output tuples to write into."""
        k = iter(out) if out is not None else None
        nxt = lambda: next(k) if k is not None else None
        res = []
        res.append(tvm.tvmattn_adaln_jvp_fwd(a["x"], a["tx"], a["a"], a["ta"], a["b"], a["tb"], eps, out=nxt()))
        res.append(tvm.tvmattn_adaln_jvp_bwd(a["x"], a["tx"], a["a"], a["ta"], a["b"], a["tb"], eps, a["gy"], a["gty"],
                                             out=nxt(), workspace=ws))
        res.append(tvm.tvmattn_gate_jvp_fwd(g["x"], g["tx"], g["h"], g["th"], g["c"], g["tc"], eps, out=nxt()))
        res.append(tvm.tvmattn_gate_jvp_bwd(g["h"], g["th"], g["c"], g["tc"], eps, g["gz"], g["gtz"], out=nxt(), workspace=ws))
        res.append(tvm.tvmattn_gelu_jvp_fwd(e["u"], e["tu"], out=nxt()))
        res.append(tvm.tvmattn_gelu_jvp_bwd(e["u"], e["tu"], e["ga"], e["gta"], out=nxt()))
        n4 = tvm.tvmattn_qknorm_jvp_fwd(q["q"], q["tq"], q["k"], q["tk"], gq, gk, eps, out=nxt())
        res.append(n4)
        f4 = tvm.tvmattn_jvp_fwd(n4[0], n4[2], q["v"], n4[1], n4[3], q["tv"], out=nxt())
        res.append(f4)
        res.append(tvm.tvmattn_jvp_bwd_qknorm(q["q"], q["tq"], q["k"], q["tk"], gq, gk, eps, *n4, q["v"], q["tv"], *f4,
                                              q["gO"], q["gTO"], out=nxt(), workspace=ws))
        res.append(tvm.tvmattn_linear_jvp_fwd(lin["x"], lin["tx"], lin["w"], lin["b"], out=nxt()))
        res.append(tvm.tvmattn_linear_jvp_bwd(lin["x"], lin["tx"], lin["w"], lin["gy"], lin["gty"], out=nxt(), workspace=ws))
        return res

    ref = calls(None)
    torch.cuda.synchronize()
    ref = [tuple(t.clone() for t in r) for r in ref]
    bufs = [tuple(torch.empty_like(t) for t in r) for r in ref]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        calls(bufs)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        calls(bufs)
    for replay in range(3):
        for r in bufs:
            for t in r:
                t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (got, want) in enumerate(zip(bufs, ref)):
            for j, (x, y) in enumerate(zip(got, want)):
                assert torch.equal(x, y), f"replay {replay}: output {j} of call {i} differs from the eager call"


@pytest.mark.parametrize("B,T,H,d,hidden", [(2, 200, 4, 72, 1152), (1, 160, 2, 128, 512)])
def test_captured_block_chain_replays_bit_for_bit(B, T, H, d, hidden):
    """The whole block chain (paper_2511_19797_amd/block.py: about fifty launches, forward and backward, its
    intermediates allocated inside the capture from the graph's memory pool) captured once and replayed: the block's
    outputs and every gradient equal the eager chain's bit for bit on every replay, with eager work in between."""
    from paper_2511_19797_amd import block
    announce(f"graph capture of the block chain B{B} T{T} H{H} d{d} hidden{hidden}")
    x, tx, mods, tmods, params, gz, gtz = wl.make_block_inputs(B, T, H, d, hidden, seed=5)
    x, tx, gz, gtz = x.cuda(), tx.cuda(), gz.cuda(), gtz.cuda()
    dm, dtm, dp = ({k: v.cuda() for k, v in m.items()} for m in (mods, tmods, params))

    def step():
        z, tz, saved = block.block_jvp_fwd(x, tx, dm, dtm, dp, H, 1e-6, 1e-6)
        g = block.block_jvp_bwd(x, tx, dm, dtm, dp, H, 1e-6, 1e-6, saved, gz, gtz)
        return [("z", z), ("tz", tz)] + sorted(g.items())

    ref = [(n, t.clone()) for n, t in step()]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        outs = step()
    for replay in range(3):
        for _, t in outs:  # eager work between the replays: the outputs are wiped with a fill kernel
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (name, got), (rname, want) in zip(outs, ref):
            assert name == rname and torch.equal(got, want), f"replay {replay}: {name} differs from the eager chain"
