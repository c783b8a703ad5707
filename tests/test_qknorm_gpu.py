"""GPU-vs-oracle parity of the QK-norm entry points (RMSNorm with gain, tangent, backward) through the
C-ABI.  Every case prints its name before touching the GPU."""
import sys

import numpy as np
import pytest
import torch

import paper_2511_19797_amd as tvm
from oracle import rmsnorm_oracle as norc
from oracle import tvmattn_oracle as aorc
from paper_2511_19797_amd import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
EPS = 1e-6


def announce(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def sides(B, H, M, N, d, dtype, seed):
    """Query-side and key-side inputs: q, tq and upstream gradients with M rows, k, tk with N rows."""
    qs = wl.make_inputs(wl.custom(B, H, M, d, dtype), seed)
    ks = wl.make_inputs(wl.custom(B, H, N, d, dtype), seed + 1)
    gq, gk = wl.make_gains(wl.custom(B, H, N, d, dtype), seed + 2)
    return dict(q=qs["q"], tq=qs["tq"], gqn=qs["gO"], gtqn=qs["gTO"], k=ks["k"], tk=ks["tk"], gkn=ks["v"], gtkn=ks["tv"],
                gain_q=gq, gain_k=gk)


def check(inp, fwd, bwd, dtype, rows=None):
    """Every element (or the listed rows of the flattened [B*H*n, d] view) against the oracle."""
    tol = pu.TOL[dtype]
    f64 = {n: wl.to_f64(t) for n, t in inp.items()}
    worst = {}
    for sd, x, tx, g, gy, gty, o in (("q", "q", "tq", "gain_q", "gqn", "gtqn", 0), ("k", "k", "tk", "gain_k", "gkn", "gtkn", 2)):
        d = f64[x].shape[-1]
        flat = lambda a: a.reshape(-1, d)
        sel = slice(None) if rows is None else rows[sd]
        y, ty = norc.rmsnorm_jvp_fwd(flat(f64[x])[sel], flat(f64[tx])[sel], f64[g], EPS)
        gx, gtx, gg = norc.rmsnorm_jvp_bwd(flat(f64[x]), flat(f64[tx]), f64[g], EPS, flat(f64[gy]), flat(f64[gty]))
        got = lambda t: flat(t.float().cpu().numpy())[sel]
        for name, a, ref in ((sd + "n", fwd[o], y), ("t" + sd + "n", fwd[o + 1], ty), ("d" + sd, bwd[o], gx[sel]),
                             ("dt" + sd, bwd[o + 1], gtx[sel])):
            worst[name] = pu.rel_err(got(a), ref)
        worst["dgain_" + sd] = pu.rel_err(bwd[4 + o // 2].cpu().numpy(), gg)
    bad = {k: v for k, v in worst.items() if not (v <= tol)}
    assert not bad, f"rel err above {tol}: {bad} (all: {worst})"
    # the gain gradient is a float32 sum of float32 terms whatever the storage type
    assert worst["dgain_q"] <= 1e-4 and worst["dgain_k"] <= 1e-4, worst
    return worst


def run(inp):
    dev = {n: t.cuda() for n, t in inp.items()}
    fwd = tvm.tvmattn_qknorm_jvp_fwd(dev["q"], dev["tq"], dev["k"], dev["tk"], dev["gain_q"], dev["gain_k"], EPS)
    bwd = tvm.tvmattn_qknorm_jvp_bwd(dev["q"], dev["tq"], dev["k"], dev["tk"], dev["gain_q"], dev["gain_k"], EPS,
                                     dev["gqn"], dev["gtqn"], dev["gkn"], dev["gtkn"])
    torch.cuda.synchronize()
    return fwd, bwd


@pytest.mark.parametrize("B,H,M,N,d,dtype", [
    (1, 1, 1, 1, 8, "bf16"), (2, 3, 77, 77, 72, "bf16"), (1, 2, 100, 260, 64, "bf16"), (2, 1, 33, 17, 128, "bf16"),
    (1, 2, 50, 50, 136, "bf16"), (1, 1, 19, 40, 256, "bf16"), (1, 1, 70, 70, 16, "bf16"),
    (2, 3, 77, 31, 40, "f32"), (1, 2, 64, 64, 4, "f32"), (1, 1, 30, 45, 100, "f32"), (1, 1, 20, 20, 256, "f32"),
    (2, 4, 2500, 2100, 72, "bf16"),   # more rows than the workgroups cover in one pass
])
def test_every_element_against_the_oracle(B, H, M, N, d, dtype):
    announce(f"qknorm B{B} H{H} M{M} N{N} d{d} {dtype}")
    inp = sides(B, H, M, N, d, dtype, 61)
    fwd, bwd = run(inp)
    worst = check(inp, fwd, bwd, dtype)
    print("   worst rel err:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)


@pytest.mark.parametrize("d,pitch,dtype", [(20, 24, "bf16"), (7, 8, "f32"), (72, 80, "bf16"), (130, 136, "bf16")])
def test_padded_rows_and_head_dims_that_end_inside_a_chunk(d, pitch, dtype):
    """Rows pitch elements apart (a 16-byte multiple) holding d of them: the last 16-byte chunk of a row is
    read and written element by element, and the padding is left alone."""
    B, H, M, N = 2, 2, 37, 50
    announce(f"qknorm strided d{d} pitch{pitch} {dtype}")
    inp = sides(B, H, M, N, d, dtype, 62)
    dev = {}
    for n, t in inp.items():
        if t.dim() == 4:
            buf = torch.full((t.shape[0], t.shape[1], t.shape[2], pitch), 7.0, dtype=t.dtype, device="cuda")
            buf[..., :d] = t.cuda()
            dev[n] = buf[..., :d]
        else:
            dev[n] = t.cuda()
    mk = lambda like: torch.full((like.shape[0], like.shape[1], like.shape[2], pitch), 7.0, dtype=like.dtype,
                                 device="cuda")
    bufs = [mk(dev["q"]), mk(dev["q"]), mk(dev["k"]), mk(dev["k"])]
    fwd = tvm.tvmattn_qknorm_jvp_fwd(dev["q"], dev["tq"], dev["k"], dev["tk"], dev["gain_q"], dev["gain_k"], EPS,
                                     out=tuple(b[..., :d] for b in bufs))
    gbufs = [mk(dev["q"]), mk(dev["q"]), mk(dev["k"]), mk(dev["k"])]
    bwd = tvm.tvmattn_qknorm_jvp_bwd(dev["q"], dev["tq"], dev["k"], dev["tk"], dev["gain_q"], dev["gain_k"], EPS,
                                     dev["gqn"], dev["gtqn"], dev["gkn"], dev["gtkn"],
                                     out=tuple(b[..., :d] for b in gbufs) + (torch.empty_like(dev["gain_q"]),
                                                                              torch.empty_like(dev["gain_k"])))
    torch.cuda.synchronize()
    check(inp, fwd, bwd, dtype)
    for b in bufs + gbufs:
        assert bool((b[..., d:] == 7.0).all()), "padding was written"


def test_bitwise_reproducible():
    inp = sides(2, 4, 900, 1100, 72, "bf16", 63)
    announce("qknorm determinism")
    a = run(inp)
    b = run(inp)
    for x, y in zip(a[0] + a[1], b[0] + b[1]):
        assert torch.equal(x, y)


def test_full_size():
    """C4's shape in the launch configuration bench.py times: every element of every output."""
    w = wl.CONFIGS["C4"]
    announce(f"qknorm full-size {w}")
    inp = sides(w.B, w.H, w.N, w.N, w.d, w.dtype, 64)
    fwd, bwd = run(inp)
    worst = check(inp, fwd, bwd, w.dtype)
    print("   worst rel err:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)


def test_chain_with_attention():
    """QK-norm -> attention with tangent -> both backwards, as the paper's block runs them, against the two
    oracles chained in float64.  The chain rounds the normalised tensors and the gradients that flow back to
    storage precision between the two steps, the oracle chain does not: same tolerance as each step alone."""
    B, H, N, d, dtype = 2, 3, 200, 72, "bf16"
    announce("qknorm + attention chain")
    inp = wl.make_inputs(wl.custom(B, H, N, d, dtype), 65)
    gq, gk = wl.make_gains(wl.custom(B, H, N, d, dtype), 66)
    dev = {n: t.cuda() for n, t in inp.items()}
    gqd, gkd = gq.cuda(), gk.cuda()
    qn, tqn, kn, tkn = tvm.tvmattn_qknorm_jvp_fwd(dev["q"], dev["tq"], dev["k"], dev["tk"], gqd, gkd, EPS)
    o, to, lse, stats = tvm.tvmattn_jvp_fwd(qn, kn, dev["v"], tqn, tkn, dev["tv"])
    dqn, dkn, dv, dtqn, dtkn, dtv = tvm.tvmattn_jvp_bwd(qn, kn, dev["v"], tqn, tkn, dev["tv"], o, to, lse, stats,
                                                        dev["gO"], dev["gTO"])
    dq, dtq, dk, dtk, dgq, dgk = tvm.tvmattn_qknorm_jvp_bwd(dev["q"], dev["tq"], dev["k"], dev["tk"], gqd, gkd, EPS,
                                                            dqn, dtqn, dkn, dtkn)
    torch.cuda.synchronize()
    f = {n: wl.to_f64(t) for n, t in inp.items()}
    g64q, g64k = wl.to_f64(gq), wl.to_f64(gk)
    rqn, rtqn = norc.rmsnorm_jvp_fwd(f["q"], f["tq"], g64q, EPS)
    rkn, rtkn = norc.rmsnorm_jvp_fwd(f["k"], f["tk"], g64k, EPS)
    ro = aorc.attn_jvp_fwd(rqn, rkn, f["v"], rtqn, rtkn, f["tv"])
    rg = aorc.attn_jvp_bwd(rqn, rkn, f["v"], rtqn, rtkn, f["tv"], f["gO"], f["gTO"])
    rdq, rdtq, rdgq = norc.rmsnorm_jvp_bwd(f["q"], f["tq"], g64q, EPS, rg[0], rg[3])
    rdk, rdtk, rdgk = norc.rmsnorm_jvp_bwd(f["k"], f["tk"], g64k, EPS, rg[1], rg[4])
    tol = pu.TOL[dtype]
    for name, got, ref in (("o", o, ro[0]), ("to", to, ro[1]), ("dq", dq, rdq), ("dtq", dtq, rdtq), ("dk", dk, rdk),
                           ("dtk", dtk, rdtk), ("dv", dv, rg[2]), ("dtv", dtv, rg[5]), ("dgain_q", dgq, rdgq),
                           ("dgain_k", dgk, rdgk)):
        e = pu.rel_err(got.float().cpu().numpy(), ref)
        assert e <= tol, (name, e)


# ---------------------------------------------------------------- both backwards in one call
def fused_and_chained(B, H, M, N, d, seed):
    """Runs norm -> attention -> (a) the two backward calls one after the other, (b) the fused call."""
    qs = wl.make_inputs(wl.custom(B, H, M, d, "bf16"), seed)
    ks = wl.make_inputs(wl.custom(B, H, N, d, "bf16"), seed + 1)
    inp = {n: (qs if n in ("q", "tq", "gO", "gTO") else ks)[n] for n in wl.NAMES}
    gq, gk = wl.make_gains(wl.custom(B, H, N, d, "bf16"), seed + 2)
    dev = {n: t.cuda() for n, t in inp.items()}
    gqd, gkd = gq.cuda(), gk.cuda()
    qn, tqn, kn, tkn = tvm.tvmattn_qknorm_jvp_fwd(dev["q"], dev["tq"], dev["k"], dev["tk"], gqd, gkd, EPS)
    o, to, lse, stats = tvm.tvmattn_jvp_fwd(qn, kn, dev["v"], tqn, tkn, dev["tv"])
    dqn, dkn, dv, dtqn, dtkn, dtv = tvm.tvmattn_jvp_bwd(qn, kn, dev["v"], tqn, tkn, dev["tv"], o, to, lse, stats,
                                                        dev["gO"], dev["gTO"])
    dq, dtq, dk, dtk, dgq, dgk = tvm.tvmattn_qknorm_jvp_bwd(dev["q"], dev["tq"], dev["k"], dev["tk"], gqd, gkd, EPS,
                                                            dqn, dtqn, dkn, dtkn)
    chained = (dq, dk, dv, dtq, dtk, dtv, dgq, dgk)
    fused = tvm.tvmattn_jvp_bwd_qknorm(dev["q"], dev["tq"], dev["k"], dev["tk"], gqd, gkd, EPS, qn, tqn, kn, tkn,
                                       dev["v"], dev["tv"], o, to, lse, stats, dev["gO"], dev["gTO"])
    torch.cuda.synchronize()
    return inp, (gq, gk), chained, fused


FUSED_NAMES = ("dq", "dk", "dv", "dtq", "dtk", "dtv", "dgain_q", "dgain_k")


def oracle_chain(inp, gains, b, h):
    f = {n: wl.to_f64(t[b, h]) for n, t in inp.items()}
    g64q, g64k = wl.to_f64(gains[0]), wl.to_f64(gains[1])
    rqn, rtqn = norc.rmsnorm_jvp_fwd(f["q"], f["tq"], g64q, EPS)
    rkn, rtkn = norc.rmsnorm_jvp_fwd(f["k"], f["tk"], g64k, EPS)
    rg = aorc.attn_jvp_bwd_head(rqn, rkn, f["v"], rtqn, rtkn, f["tv"], f["gO"], f["gTO"])
    rdq, rdtq, rdgq = norc.rmsnorm_jvp_bwd(f["q"], f["tq"], g64q, EPS, rg[0], rg[3])
    rdk, rdtk, rdgk = norc.rmsnorm_jvp_bwd(f["k"], f["tk"], g64k, EPS, rg[1], rg[4])
    return (rdq, rdk, rg[2], rdtq, rdtk, rg[5]), (rdgq, rdgk)


@pytest.mark.parametrize("B,H,M,N,d", [
    (1, 2, 100, 100, 16), (2, 1, 130, 70, 32), (1, 1, 97, 200, 48), (1, 2, 200, 200, 64), (2, 3, 200, 260, 72),
    (1, 1, 65, 193, 96), (1, 1, 1, 1, 8), (1, 2, 300, 40, 40),
])
def test_fused_backward_against_the_oracle_chain_and_the_two_calls(B, H, M, N, d):
    announce(f"fused attention + qknorm backward B{B} H{H} M{M} N{N} d{d}")
    inp, gains, chained, fused = fused_and_chained(B, H, M, N, d, 71)
    # against the two calls made one after the other: the same arithmetic on the same rounded gradients, so the six
    # tensors agree to the last bit; the gain gradients add the same terms in another order
    for name, a, b in zip(FUSED_NAMES[:6], chained, fused):
        assert torch.equal(a, b), name
    for name, a, b in zip(FUSED_NAMES[6:], chained[6:], fused[6:]):
        assert pu.rel_err(b.cpu().numpy(), a.cpu().numpy().astype(np.float64)) <= 1e-5, name
    # against the float64 chain of the two oracles, every head
    gsum = [np.zeros(d), np.zeros(d)]
    for b in range(B):
        for h in range(H):
            ref, rg = oracle_chain(inp, gains, b, h)
            for name, got, r in zip(FUSED_NAMES[:6], fused, ref):
                e = pu.rel_err(got[b, h].float().cpu().numpy(), r)
                assert e <= pu.TOL["bf16"], (name, b, h, e)
            gsum[0] += rg[0]
            gsum[1] += rg[1]
    for name, got, r in zip(FUSED_NAMES[6:], fused[6:], gsum):
        assert pu.rel_err(got.cpu().numpy(), r) <= pu.TOL["bf16"], name


def test_fused_backward_full_size():
    """C4 in the launch configuration bench.py times: bitwise against the two separate calls for the tensors,
    sampled heads against the oracle chain."""
    w = wl.CONFIGS["C4"]
    announce(f"fused attention + qknorm backward, full size {w}")
    inp, gains, chained, fused = fused_and_chained(w.B, w.H, w.N, w.N, w.d, 72)
    for name, a, b in zip(FUSED_NAMES[:6], chained, fused):
        assert torch.equal(a, b), name
    for name, a, b in zip(FUSED_NAMES[6:], chained[6:], fused[6:]):
        assert pu.rel_err(b.cpu().numpy(), a.cpu().numpy().astype(np.float64)) <= 1e-5, name
    for (b, h) in ((0, 0), (w.B - 1, w.H - 1)):
        ref, _ = oracle_chain(inp, gains, b, h)
        for name, got, r in zip(FUSED_NAMES[:6], fused, ref):
            e = pu.rel_err(got[b, h].float().cpu().numpy(), r)
            assert e <= pu.TOL["bf16"], (name, b, h, e)


def test_fused_backward_refuses_what_it_does_not_serve():
    """float32 and head dims above 96 are answered with status -2 and a zero workspace size, nothing launched."""
    for B, H, N, d, dtype in ((1, 1, 64, 128, "bf16"), (1, 1, 64, 32, "f32")):
        announce(f"fused backward unsupported d{d} {dtype}")
        x = wl.make_inputs(wl.custom(B, H, N, d, dtype), 73)["q"].cuda()
        g = torch.ones(d, dtype=torch.float32, device="cuda")
        assert tvm.tvmattn_jvp_bwd_qknorm_workspace_bytes(x) == 0
        row = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
        with pytest.raises(tvm.TvmattnError) as ei:
            tvm.tvmattn_jvp_bwd_qknorm(x, x, x, x, g, g, EPS, x, x, x, x, x, x, x, x, row, row, x, x)
        assert ei.value.status == -2


# ---------------------------------------------------------------- norm and attention forward in one call
FWD_NAMES = ("qn", "tqn", "kn", "tkn", "o", "to", "lse", "stats")


def fused_forward_and_two_calls(B, H, M, N, d, seed, scale=0.0):
    qs = wl.make_inputs(wl.custom(B, H, M, d, "bf16"), seed)
    ks = wl.make_inputs(wl.custom(B, H, N, d, "bf16"), seed + 1)
    inp = {n: (qs if n in ("q", "tq", "gO", "gTO") else ks)[n] for n in wl.NAMES}
    gq, gk = wl.make_gains(wl.custom(B, H, N, d, "bf16"), seed + 2)
    dev = {n: t.cuda() for n, t in inp.items()}
    gqd, gkd = gq.cuda(), gk.cuda()
    n4 = tvm.tvmattn_qknorm_jvp_fwd(dev["q"], dev["tq"], dev["k"], dev["tk"], gqd, gkd, EPS)
    f4 = tvm.tvmattn_jvp_fwd(n4[0], n4[2], dev["v"], n4[1], n4[3], dev["tv"], scale=scale)
    fused = tvm.tvmattn_jvp_fwd_qknorm(dev["q"], dev["tq"], dev["k"], dev["tk"], gqd, gkd, EPS, dev["v"], dev["tv"], scale=scale)
    torch.cuda.synchronize()
    return inp, (gq, gk), tuple(n4) + tuple(f4), fused


def check_fused_forward(inp, gains, two, fused, heads, scale=None):
    # the key side runs through the same kernel either way
    assert torch.equal(two[2], fused[2]) and torch.equal(two[3], fused[3])
    # against the two calls: the same formulas in float32 in another order, then one bf16 rounding of qn, tqn
    for name, a, b in zip(FWD_NAMES, two, fused):
        e = pu.rel_err(b.float().cpu().numpy(), a.float().cpu().numpy().astype(np.float64))
        assert e <= 1e-2, (name, e)
    g64q, g64k = wl.to_f64(gains[0]), wl.to_f64(gains[1])
    for (b, h) in heads:
        f = {n: wl.to_f64(t[b, h]) for n, t in inp.items()}
        rqn, rtqn = norc.rmsnorm_jvp_fwd(f["q"], f["tq"], g64q, EPS)
        rkn, rtkn = norc.rmsnorm_jvp_fwd(f["k"], f["tk"], g64k, EPS)
        ro, rto, rlse, rstats = aorc.attn_jvp_fwd_head(rqn, rkn, f["v"], rtqn, rtkn, f["tv"], scale)
        for name, got, r in zip(FWD_NAMES, fused, (rqn, rtqn, rkn, rtkn, ro, rto, rlse, rstats)):
            g = got[b, h].float().cpu().numpy()
            # (lse and stats are sums of O(1) scores: with a single key they are one score, whose error is that of a
            # dot product of bf16-rounded rows, absolute, however small the score)
            e = float(np.abs(g - r).max()) / max(1.0, float(np.abs(r).max())) if name in ("lse", "stats") else pu.rel_err(g, r)
            assert e <= pu.TOL["bf16"], (name, b, h, e)


@pytest.mark.parametrize("B,H,M,N,d", [
    (1, 2, 100, 100, 16), (2, 1, 130, 70, 32), (1, 1, 97, 200, 48), (1, 2, 200, 200, 64), (2, 3, 200, 260, 72),
    (1, 1, 65, 193, 96), (1, 1, 1, 1, 8), (1, 2, 300, 40, 40), (1, 1, 70, 150, 128), (1, 1, 33, 90, 104),
    (1, 2, 300, 600, 72),   # eight-wave workgroups (512 keys or more, more than 128 queries), ragged in both
    (1, 1, 257, 513, 64), (1, 1, 512, 1000, 96), (1, 1, 129, 512, 24),
])
def test_fused_forward_against_the_oracle_chain_and_the_two_calls(B, H, M, N, d):
    announce(f"qknorm + attention forward in one call B{B} H{H} M{M} N{N} d{d}")
    inp, gains, two, fused = fused_forward_and_two_calls(B, H, M, N, d, 81)
    check_fused_forward(inp, gains, two, fused, [(b, h) for b in range(B) for h in range(H)])


def test_fused_forward_explicit_scale_and_nothing_saved():
    announce("qknorm + attention forward in one call: explicit scale, save=False")
    B, H, M, N, d = 1, 2, 150, 220, 72
    inp, gains, two, fused = fused_forward_and_two_calls(B, H, M, N, d, 82, scale=0.2)
    check_fused_forward(inp, gains, two, fused, [(0, 0), (0, 1)], scale=0.2)
    dev = {n: t.cuda() for n, t in inp.items()}
    out = tvm.tvmattn_jvp_fwd_qknorm(dev["q"], dev["tq"], dev["k"], dev["tk"], gains[0].cuda(), gains[1].cuda(), EPS,
                                     dev["v"], dev["tv"], scale=0.2, save=False)
    torch.cuda.synchronize()
    assert out[6] is None and out[7] is None
    for name, a, b in zip(FWD_NAMES[:6], fused, out):
        assert torch.equal(a, b), name


def test_fused_forward_full_size_and_the_backward_takes_its_outputs():
    """C4 in the launch configuration bench.py times; sampled heads against the oracle chain; the rows it leaves
    behind feed the fused backward, whose gradients are compared with those from the two forward calls' rows."""
    w = wl.CONFIGS["C4"]
    announce(f"qknorm + attention forward in one call, full size {w}")
    inp, gains, two, fused = fused_forward_and_two_calls(w.B, w.H, w.N, w.N, w.d, 83)
    check_fused_forward(inp, gains, two, fused, [(0, 0), (w.B - 1, w.H - 1)])
    dev = {n: t.cuda() for n, t in inp.items()}
    gq, gk = gains[0].cuda(), gains[1].cuda()
    bwd = lambda f: tvm.tvmattn_jvp_bwd_qknorm(dev["q"], dev["tq"], dev["k"], dev["tk"], gq, gk, EPS, f[0], f[1], f[2], f[3],
                                               dev["v"], dev["tv"], f[4], f[5], f[6], f[7], dev["gO"], dev["gTO"])
    ga, gb = bwd(two), bwd(fused)
    torch.cuda.synchronize()
    for name, a, b in zip(FUSED_NAMES, ga, gb):
        e = pu.rel_err(b.float().cpu().numpy(), a.float().cpu().numpy().astype(np.float64))
        assert e <= 1e-2, (name, e)


def test_fused_forward_refuses_what_it_does_not_serve():
    for B, H, N, d, dtype in ((1, 1, 64, 32, "f32"), (1, 1, 64, 136, "bf16")):
        announce(f"fused forward unsupported d{d} {dtype}")
        x = wl.make_inputs(wl.custom(B, H, N, d, dtype), 84)["q"].cuda()
        g = torch.ones(d, dtype=torch.float32, device="cuda")
        with pytest.raises(tvm.TvmattnError) as ei:
            tvm.tvmattn_jvp_fwd_qknorm(x, x, x, x, g, g, EPS, x, x)
        assert ei.value.status == -2
