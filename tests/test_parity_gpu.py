"""GPU-vs-oracle parity through the C-ABI (ctypes binding).  Every case prints its name
before touching the GPU so a failing run names its case."""
import sys

import numpy as np
import pytest
import torch

import paper_2511_19797_amd as tvm
from paper_2511_19797_amd import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def announce(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def run_case(w, seed, heads=None, scale=0.0, force_generic=False):
    announce(f"{w} seed={seed} scale={scale} generic={force_generic}")
    inp = wl.make_inputs(w, seed)
    fwd, grads = pu.run_gpu(inp, scale, flags=tvm.TVMATTN_FLAG_PLAIN_ALU if force_generic else 0)
    heads = pu.all_heads(w) if heads is None else heads
    pu.check_heads(w, inp, fwd, grads, heads, scale=(scale or None))
    return inp, fwd, grads


# ---------------------------------------------------------------- float32 (plain-ALU kernels)
def test_c1_f32_tiny():
    run_case(wl.CONFIGS["C1"], seed=1)


@pytest.mark.parametrize("B,H,N,d", [(2, 3, 77, 40), (1, 2, 1, 8), (1, 1, 130, 256), (1, 2, 64, 4), (2, 1, 200, 72)])
def test_f32_ragged_shapes(B, H, N, d):
    run_case(wl.custom(B, H, N, d, "f32"), seed=2)


def test_f32_explicit_scale():
    run_case(wl.custom(1, 2, 50, 16, "f32"), seed=3, scale=0.3)


# ---------------------------------------------------------------- bf16 on the plain-ALU kernels
@pytest.mark.parametrize("B,H,N,d", [(1, 2, 96, 64), (2, 2, 70, 136), (1, 1, 33, 72)])
def test_bf16_generic_kernels(B, H, N, d):
    run_case(wl.custom(B, H, N, d, "bf16"), seed=4, force_generic=True)


# ---------------------------------------------------------------- bf16 matrix-core kernels, small
@pytest.mark.parametrize("B,H,N,d", [
    (2, 2, 256, 64),    # C2 shape, few heads
    (2, 2, 256, 72),    # C3 shape, few heads: padded head dim
    (1, 3, 200, 72),    # ragged tail in both the last key tile and the last query tile
    (1, 2, 65, 72),     # one full tile plus one row
    (1, 2, 1, 64),      # single token
    (1, 2, 31, 8),      # smallest head dim, less than one tile
    (2, 1, 300, 128),   # C5 head dim, ragged
    (1, 2, 129, 40), (1, 1, 257, 96), (1, 1, 130, 32), (1, 1, 100, 16), (1, 1, 192, 80), (1, 1, 64, 104),
    (1, 1, 160, 120),
])
def test_bf16_mfma_small(B, H, N, d):
    run_case(wl.custom(B, H, N, d, "bf16"), seed=5)


@pytest.mark.parametrize("d", [8, 24, 40, 64, 72, 96])
def test_bf16_hand_scheduled_tile_boundaries(d):
    """Every instantiation of the hand-scheduled backward kernels (one per padded head dim) at the
    sequence lengths where their tile pipeline changes shape: less than a tile, exactly one, two
    and three tiles (the three LDS stages wrap), one row more or fewer, a workgroup boundary."""
    for N in (17, 63, 64, 65, 127, 128, 129, 191, 192, 193, 320):
        run_case(wl.custom(1, 1, N, d, "bf16"), seed=20 + N % 7)


@pytest.mark.parametrize("d", [104, 112, 120, 128])
def test_bf16_hand_scheduled_passes_tile_boundaries(d):
    """Head dims above 96: with more than 64 keys the query side of the backward runs as one hand-scheduled pass over
    tiles of 32 keys, with more than 64 queries the key side as two such passes over tiles of 32 queries (both
    instantiations: contraction padded to 112 and to 128).  Sequence lengths where that pipeline changes shape: the
    last length on the generic-order kernels and the first one on the passes, three and four tiles (the three LDS
    stages wrap), one row more or fewer, a workgroup boundary of 128 rows, several workgroups per head; then M != N
    either way round, with a ragged last tile on both sides, and with one side short enough for its generic-order
    kernel next to the other side's passes (the row vectors change convention).  Every element of all ten outputs."""
    import dataclasses
    for N in (64, 65, 95, 96, 97, 127, 128, 129, 161, 320):
        run_case(wl.custom(1, 1, N, d, "bf16"), seed=30 + N % 7)
    for M, N in ((65, 300), (300, 65), (130, 129), (40, 200), (200, 40)):
        w = dataclasses.replace(wl.custom(1, 2, N, d, "bf16"), M=M)
        run_case(w, seed=40 + M % 13)


@pytest.mark.parametrize("d", [8, 24, 40, 64, 72, 96])
def test_bf16_wide_forward_workgroups(d):
    """From 512 keys on (head dims up to 96, more than 128 queries) the forward runs eight-wave workgroups of 256
    query rows.  Every instantiation of it (one per padded head dim), with a whole and a ragged last key block,
    with workgroups whose upper waves hold no query row (M = 257, 300), and with M != N either way round: every
    element of all ten outputs against the oracle."""
    import dataclasses
    for N in (512, 513, 543, 1000):
        run_case(wl.custom(1, 2 if N == 512 else 1, N, d, "bf16"), seed=60 + N % 11)
    for M, N in ((257, 512), (300, 543), (700, 600), (600, 700)):
        w = dataclasses.replace(wl.custom(1, 1, N, d, "bf16"), M=M)
        run_case(w, seed=70 + M % 13)


def test_inputs_sliced_from_a_fused_projection():
    """q, k, v (and the tangents, and the upstream gradients) sliced out of fused [B,N,3,H,D] buffers: not dense, so
    the outputs must be allocated with the inputs' strides.  Forward and backward against the oracle, matrix-core
    and plain-ALU paths."""
    for dtype, d, N in (("bf16", 72, 200), ("bf16", 64, 520), ("bf16", 128, 200), ("f32", 24, 70)):
        w = wl.custom(2, 3, N, d, dtype)
        announce(f"fused-QKV slices {w}")
        inp = wl.make_inputs(w, 15)
        def fused(a, b, c):  # [B,H,N,D] x 3 -> one [B,N,3,H,D] buffer and its three [B,H,N,D] views
            buf = torch.stack([a, b, c], dim=0).permute(1, 3, 0, 2, 4).contiguous().cuda()
            return [buf[:, :, i].permute(0, 2, 1, 3) for i in range(3)]
        q, k, v = fused(inp["q"], inp["k"], inp["v"])
        tq, tk, tv = fused(inp["tq"], inp["tk"], inp["tv"])
        gO, gTO, _ = fused(inp["gO"], inp["gTO"], inp["gO"])
        assert not q.is_contiguous() and q.stride() == (N * 3 * 3 * d, d, 3 * 3 * d, 1)
        o, to, lse, stats = tvm.tvmattn_jvp_fwd(q, k, v, tq, tk, tv)
        assert o.stride() == q.stride()
        grads = tvm.tvmattn_jvp_bwd(q, k, v, tq, tk, tv, o, to, lse, stats, gO, gTO)
        torch.cuda.synchronize()
        assert grads[0].stride() == q.stride() and grads[1].stride() == k.stride()
        pu.check_heads(w, inp, (o, to, lse, stats), grads, pu.all_heads(w))


def test_bf16_mfma_scaled_inputs():
    # C4's small tangents and C5's sharpened keys at a size the oracle does in full
    run_case(wl.custom(1, 2, 384, 72, "bf16", tangent_std=0.1), seed=6)
    run_case(wl.custom(1, 2, 512, 128, "bf16", key_scale=2.0), seed=7)
    run_case(wl.custom(1, 2, 128, 64, "bf16"), seed=8, scale=0.2)


def test_strided_layout_bnhd():
    """Tensors stored [B,N,H,D] and viewed as [B,H,N,D] (what a fused QKV projection hands over)."""
    for dtype, d in (("bf16", 72), ("bf16", 112), ("f32", 24)):
        w = wl.custom(2, 3, 150, d, dtype)
        announce(f"strided {w}")
        inp = wl.make_inputs(w, 9)
        dev = {n: t.cuda().permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for n, t in inp.items()}
        assert dev["q"].stride(1) == d and dev["q"].stride(2) == 3 * d
        o, to, lse, stats = tvm.tvmattn_jvp_fwd(*(dev[n] for n in wl.NAMES[:6]))
        grads = tvm.tvmattn_jvp_bwd(*(dev[n] for n in wl.NAMES[:6]), o, to, lse, stats, dev["gO"], dev["gTO"])
        torch.cuda.synchronize()
        assert o.stride() == dev["q"].stride()
        pu.check_heads(w, inp, (o, to, lse, stats), grads, pu.all_heads(w))


def test_strided_layout_with_more_queries_than_keys():
    """Query side stored [B,M,H,D], key side contiguous [B,H,N,D], M != N: the two sides have their own strides."""
    import dataclasses
    for dtype, d in (("bf16", 72), ("bf16", 128), ("f32", 24)):
        w = dataclasses.replace(wl.custom(2, 3, 90, d, dtype), M=150)
        announce(f"strided, M != N {w}")
        inp = wl.make_inputs(w, 10)
        dev = {n: (t.cuda().permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) if n in ("q", "tq", "gO", "gTO")
                   else t.cuda()) for n, t in inp.items()}
        assert dev["q"].stride(2) == 3 * d and dev["k"].stride(2) == d and dev["q"].shape[2] == 150
        o, to, lse, stats = tvm.tvmattn_jvp_fwd(*(dev[n] for n in wl.NAMES[:6]))
        grads = tvm.tvmattn_jvp_bwd(*(dev[n] for n in wl.NAMES[:6]), o, to, lse, stats, dev["gO"], dev["gTO"])
        torch.cuda.synchronize()
        assert o.stride() == dev["q"].stride() and grads[1].stride() == dev["k"].stride()
        pu.check_heads(w, inp, (o, to, lse, stats), grads, pu.all_heads(w))


@pytest.mark.parametrize("d", [72, 128])
def test_bitwise_reproducible(d):
    w = wl.custom(2, 2, 333, d, "bf16")
    announce(f"determinism {w}")
    inp = wl.make_inputs(w, 10)
    f1, g1 = pu.run_gpu(inp)
    f2, g2 = pu.run_gpu(inp)
    for a, b in zip(list(f1) + list(g1), list(f2) + list(g2)):
        assert torch.equal(a, b)


@pytest.mark.parametrize("d", [72, 120])
def test_zero_tangents_and_zero_grads_on_gpu(d):
    w = wl.custom(1, 2, 100, d, "bf16")
    announce(f"zero tangents {w}")
    inp = wl.make_inputs(w, 11)
    for n in ("tq", "tk", "tv"):
        inp[n].zero_()
    fwd, grads = pu.run_gpu(inp)
    assert float(fwd[1].float().abs().max()) == 0.0 and float(fwd[3].abs().max()) == 0.0
    pu.check_heads(w, inp, fwd, grads, pu.all_heads(w))


def test_growing_scores_force_rescales():
    """Keys whose scores keep growing along the sequence: the forward's reference maximum has to be
    raised (and its accumulators rescaled) many times, and the backward sees sharply peaked rows."""
    w = wl.custom(1, 2, 512, 72, "bf16")
    announce(f"growing scores {w}")
    inp = wl.make_inputs(w, 13)
    ramp = torch.linspace(0.2, 6.0, w.N).view(1, 1, w.N, 1)
    inp["k"] = (inp["k"].float() * ramp + inp["q"].float().mean(dim=2, keepdim=True) * ramp).to(torch.bfloat16)
    fwd, grads = pu.run_gpu(inp)
    pu.check_heads(w, inp, fwd, grads, pu.all_heads(w))


def test_backward_is_linear_in_upstream_gradients():
    """bwd(a gO1 + gO2, a gTO1 + gTO2) = a bwd(gO1, gTO1) + bwd(gO2, gTO2) up to bf16 rounding of the
    outputs; with power-of-two a and the second pair zero it is exact scaling."""
    _backward_scales_exactly(72)


def test_backward_is_linear_in_upstream_gradients_wide_heads():
    _backward_scales_exactly(128)


def _backward_scales_exactly(d):
    w = wl.custom(1, 2, 200, d, "bf16")
    announce(f"linearity {w}")
    inp = wl.make_inputs(w, 14)
    fwd, g1 = pu.run_gpu(inp)
    inp2 = dict(inp)
    inp2["gO"] = (inp["gO"].float() * 4.0).to(torch.bfloat16)
    inp2["gTO"] = (inp["gTO"].float() * 4.0).to(torch.bfloat16)
    _, g4 = pu.run_gpu(inp2)
    for a, b in zip(g1, g4):
        assert torch.equal((a.float() * 4.0).to(torch.bfloat16), b)


def _chunked_oracle_bwd(a, rows_per_chunk=512):
    """The oracle's backward of one head, one block of query rows at a time: softmax rows are
    independent, so the query gradients of a block are exact and the key-side gradients are the sums
    of the blocks' contributions.  Keeps the N x N matrices out of memory."""
    q, k, v, tq, tk, tv, gO, gTO = a
    N = q.shape[0]
    dq, dtq = np.zeros_like(q), np.zeros_like(q)
    dk, dv, dtk, dtv = (np.zeros_like(k) for _ in range(4))
    for r0 in range(0, N, rows_per_chunk):
        r = slice(r0, min(N, r0 + rows_per_chunk))
        g = pu.orc.attn_jvp_bwd_head(q[r], k, v, tq[r], tk, tv, gO[r], gTO[r])
        dq[r], dtq[r] = g[0], g[3]
        dk += g[1]
        dv += g[2]
        dtk += g[4]
        dtv += g[5]
    return dq, dk, dv, dtq, dtk, dtv


# ---------------------------------------------------------------- the five configs at full size
def _column_sums_vanish(w, grads):
    """Holds for every head at any size: adding one vector to all keys of a head changes neither O nor tO, so the
    key gradients and the key-tangent gradients sum to zero over the keys (up to the bf16 rounding of each of
    the N summands)."""
    dq, dk, dv, dtq, dtk, dtv = grads
    for g in (dk, dtk):
        col_sum = g.float().sum(dim=2).abs().max()
        bound = 4.0 * (2.0 ** -8) * g.float().abs().max() * (w.N ** 0.5)
        assert float(col_sum) <= float(bound), (float(col_sum), float(bound))


@pytest.mark.parametrize("name", ["C2", "C3", "C4", "X3", "X4", "XA"])
def test_full_size_configs_all_heads(name):
    """Full B,H,N,d in the launch configuration bench.py times: every element of all ten outputs of EVERY
    (batch, head) against the oracle."""
    w = wl.CONFIGS[name]
    announce(f"full-size, all {w.heads} heads: {w}")
    inp = wl.make_inputs(w, 100 + (int(name[1]) if name[1].isdigit() else 20) + (10 if name[0] == "X" else 0))
    fwd, grads = pu.run_gpu(inp)
    for t in list(fwd) + list(grads):
        assert bool(torch.isfinite(t.float()).all())
    pu.check_heads(w, inp, fwd, grads, pu.all_heads(w))
    _column_sums_vanish(w, grads)


def test_full_size_c5_all_heads():
    """C5 (N = 4096, d = 128, keys x 2) at full size, all 48 heads: the oracle works through a head in blocks of
    query rows (softmax rows are independent), which keeps its N x N matrices at 512 x 4096."""
    w = wl.CONFIGS["C5"]
    announce(f"full-size, all {w.heads} heads: {w}")
    inp = wl.make_inputs(w, 105)
    fwd, grads = pu.run_gpu(inp)
    for t in list(fwd) + list(grads):
        assert bool(torch.isfinite(t.float()).all())
    got_host = [t.float().cpu().numpy() for t in list(fwd) + list(grads)]
    worst, worst_elem = {}, {}
    for n_done, (b, h) in enumerate(pu.all_heads(w)):
        a = [wl.to_f64(inp[n][b, h]) for n in wl.NAMES]
        ref_f = [np.concatenate(x) for x in zip(*[
            pu.orc.attn_jvp_fwd_head(a[0][r0:r0 + 1024], a[1], a[2], a[3][r0:r0 + 1024], a[4], a[5])
            for r0 in range(0, w.N, 1024)])]
        ref_g = _chunked_oracle_bwd(a)
        for nm, got, ref in zip(pu.FWD_NAMES + pu.BWD_NAMES, got_host, list(ref_f) + list(ref_g)):
            worst[nm] = max(worst.get(nm, 0.0), pu.rel_err(got[b, h], ref))
            worst_elem[nm] = max(worst_elem.get(nm, 0.0), pu.elem_err(got[b, h], ref))
        if n_done % 8 == 7:
            print(f"   {n_done + 1} heads compared", flush=True)
    print("   max|err|/max|ref|      :", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)
    print("   max |err|/(|ref|+rms)  :", {k: f"{v:.2e}" for k, v in worst_elem.items()}, flush=True)
    bad = {k: v for k, v in worst.items() if not (v <= pu.TOL["bf16"])}
    assert not bad, bad
    _column_sums_vanish(w, grads)


# ---------------------------------------------------------------- long sequences (the paper's kernel-benchmark shapes)
def test_long_sequence_whole_head():
    """N = 8192 (128 tiles; every LDS stage reused 40 times), one head of 64: every element of all ten
    outputs against the oracle, which works through the head in blocks of query rows."""
    w = wl.custom(1, 1, 8192, 64, "bf16")
    announce(f"long sequence {w}")
    inp = wl.make_inputs(w, 31)
    fwd, grads = pu.run_gpu(inp)
    a = [wl.to_f64(inp[n][0, 0]) for n in wl.NAMES]
    ref_f = [np.concatenate(x) for x in zip(*[
        pu.orc.attn_jvp_fwd_head(a[0][r0:r0 + 1024], a[1], a[2], a[3][r0:r0 + 1024], a[4], a[5])
        for r0 in range(0, w.N, 1024)])]
    ref_g = _chunked_oracle_bwd(a)
    worst, worst_elem = {}, {}
    for name, got, ref in list(zip(pu.FWD_NAMES, fwd, ref_f)) + list(zip(pu.BWD_NAMES, grads, ref_g)):
        worst[name] = pu.rel_err(got[0, 0].float().cpu().numpy(), ref)
        worst_elem[name] = pu.elem_err(got[0, 0].float().cpu().numpy(), ref)
    print("   max|err|/max|ref|      :", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)
    print("   max |err|/(|ref|+rms)  :", {k: f"{v:.2e}" for k, v in worst_elem.items()}, flush=True)
    bad = {k: v for k, v in worst.items() if not (v <= pu.TOL["bf16"])}
    assert not bad, bad


def test_longest_benchmark_shape_sampled_rows():
    """N = 32768, the longest sequence of the paper's kernel benchmark (2 heads of 64): the oracle checks
    o, to, lse, stats, dq and dtq on a seeded sample of query rows (all of them row-local), the key-side
    gradients through the properties that hold at any size."""
    w = wl.custom(1, 2, 32768, 64, "bf16")
    announce(f"longest benchmark shape {w}")
    inp = wl.make_inputs(w, 32)
    fwd, grads = pu.run_gpu(inp)
    for t in list(fwd) + list(grads):
        assert bool(torch.isfinite(t.float()).all())
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 127, 128, w.N - 1], rng.integers(0, w.N, 252)]))
    dq, dk, dv, dtq, dtk, dtv = grads
    for h in range(w.H):
        a = [wl.to_f64(inp[n][0, h]) for n in wl.NAMES]
        ro = pu.orc.attn_jvp_fwd_head(a[0][rows], a[1], a[2], a[3][rows], a[4], a[5])
        rg = pu.orc.attn_jvp_bwd_head(a[0][rows], a[1], a[2], a[3][rows], a[4], a[5], a[6][rows], a[7][rows])
        # the row sample's maxima stand in for the tensors' (rel_err scales by the reference's maximum)
        for name, got, ref in list(zip(pu.FWD_NAMES, fwd, ro)) + [("dq", dq, rg[0]), ("dtq", dtq, rg[3])]:
            e = pu.rel_err(got[0, h].float().cpu().numpy()[rows], ref)
            assert e <= pu.TOL["bf16"], (name, h, e)
    for g in (dk, dtk):
        col_sum = g.float().sum(dim=2).abs().max()
        bound = 4.0 * (2.0 ** -8) * g.float().abs().max() * (w.N ** 0.5)
        assert float(col_sum) <= float(bound), (float(col_sum), float(bound))


# ---------------------------------------------------------------- one upstream gradient only
@pytest.mark.parametrize("B,H,N,d,dtype", [
    (1, 2, 100, 16, "bf16"), (2, 1, 200, 64, "bf16"), (1, 2, 320, 72, "bf16"), (1, 1, 193, 96, "bf16"),
    (1, 1, 257, 128, "bf16"), (1, 2, 70, 136, "bf16"), (1, 2, 64, 32, "f32"),
    (1, 2, 130, 32, "bf16"), (1, 1, 97, 48, "bf16"), (1, 1, 64, 80, "bf16"), (2, 1, 33, 8, "bf16"), (1, 1, 2, 40, "bf16"),
    # head dims above 96: the tangent path's key side as two passes (more than 64 queries) and in one (64)
    (1, 2, 97, 112, "bf16"), (1, 1, 65, 104, "bf16"), (1, 1, 64, 120, "bf16"), (2, 1, 160, 128, "bf16"),
])
def test_one_sided_backward(B, H, N, d, dtype):
    """gTO = None is the ordinary attention backward (the oracle with a zero gTO; tangent tensors not
    even passed), gO = None the tangent path alone (the oracle with a zero gO); a forward that saves
    nothing returns the same o, to bit for bit."""
    w = wl.custom(B, H, N, d, dtype)
    announce(f"one-sided {w}")
    inp = wl.make_inputs(w, 41)
    dev = {n: t.cuda() for n, t in inp.items()}
    six = [dev[n] for n in wl.NAMES[:6]]
    o, to, lse, stats = tvm.tvmattn_jvp_fwd(*six)
    o2, to2, none1, none2 = tvm.tvmattn_jvp_fwd(*six, save=False)
    assert none1 is None and none2 is None and torch.equal(o, o2) and torch.equal(to, to2)
    g_only = tvm.tvmattn_jvp_bwd(six[0], six[1], six[2], None, None, None, o, None, lse, None, dev["gO"], None)
    assert g_only[3] is None and g_only[4] is None and g_only[5] is None
    t_only = tvm.tvmattn_jvp_bwd(*six, o, to, lse, stats, None, dev["gTO"])
    torch.cuda.synchronize()
    tol = pu.TOL[dtype]
    for b in range(B):
        for h in range(H):
            a = [wl.to_f64(inp[n][b, h]) for n in wl.NAMES]
            zero = np.zeros_like(a[6])
            ref_g = pu.orc.attn_jvp_bwd_head(*a[:6], a[6], zero)
            ref_t = pu.orc.attn_jvp_bwd_head(*a[:6], zero, a[7])
            for name, got, ref in zip(pu.BWD_NAMES[:3], g_only[:3], ref_g[:3]):
                e = pu.rel_err(got[b, h].float().cpu().numpy(), ref)
                assert e <= tol, ("gO only", name, b, h, e)
            for name, got, ref in zip(pu.BWD_NAMES, t_only, ref_t):
                e = pu.rel_err(got[b, h].float().cpu().numpy(), ref)
                assert e <= tol, ("gTO only", name, b, h, e)


def test_one_sided_backward_full_size():
    """C4 in the launch configurations bench.py reports for the two one-sided backwards: sampled heads
    against the oracle, key-gradient column sums for all."""
    w = wl.CONFIGS["C4"]
    announce(f"one-sided full-size {w}")
    inp = wl.make_inputs(w, 104)
    dev = {n: t.cuda() for n, t in inp.items()}
    six = [dev[n] for n in wl.NAMES[:6]]
    o, to, lse, stats = tvm.tvmattn_jvp_fwd(*six)
    dq, dk, dv, _, _, _ = tvm.tvmattn_jvp_bwd(six[0], six[1], six[2], None, None, None, o, None, lse, None,
                                              dev["gO"], None)
    torch.cuda.synchronize()
    for t in (dq, dk, dv):
        assert bool(torch.isfinite(t.float()).all())
    for (b, h) in ((0, 0), (w.B - 1, w.H - 1), (7, 3)):
        a = [wl.to_f64(inp[n][b, h]) for n in wl.NAMES]
        ref = pu.orc.attn_jvp_bwd_head(*a[:6], a[6], np.zeros_like(a[6]))
        for name, got, r in zip(pu.BWD_NAMES[:3], (dq, dk, dv), ref[:3]):
            e = pu.rel_err(got[b, h].float().cpu().numpy(), r)
            assert e <= pu.TOL["bf16"], (name, b, h, e)
    col_sum = dk.float().sum(dim=2).abs().max()
    assert float(col_sum) <= 4.0 * (2.0 ** -8) * float(dk.float().abs().max()) * (w.N ** 0.5)
    # the tangent path alone (Steps 1-6 of App. C by themselves), same launch configuration
    t_only = tvm.tvmattn_jvp_bwd(*six, o, to, lse, stats, None, dev["gTO"])
    torch.cuda.synchronize()
    for t in t_only:
        assert bool(torch.isfinite(t.float()).all())
    for (b, h) in ((0, 0), (w.B - 1, w.H - 1), (5, 11)):
        a = [wl.to_f64(inp[n][b, h]) for n in wl.NAMES]
        ref = pu.orc.attn_jvp_bwd_head(*a[:6], np.zeros_like(a[6]), a[7])
        for name, got, r in zip(pu.BWD_NAMES, t_only, ref):
            e = pu.rel_err(got[b, h].float().cpu().numpy(), r)
            assert e <= pu.TOL["bf16"], ("gTO only", name, b, h, e)
    for g in (t_only[1], t_only[4]):  # the rows of gZ and gZt sum to zero, so dK and dtK sum to zero over the keys
        col_sum = g.float().sum(dim=2).abs().max()
        assert float(col_sum) <= 4.0 * (2.0 ** -8) * float(g.float().abs().max()) * (w.N ** 0.5)


# ---------------------------------------------------------------- M queries, N keys
@pytest.mark.parametrize("B,H,M,N,d,dtype", [
    (1, 2, 100, 260, 72, "bf16"), (2, 1, 300, 64, 64, "bf16"), (1, 1, 1, 70, 16, "bf16"), (1, 2, 129, 17, 32, "bf16"),
    (1, 1, 65, 193, 96, "bf16"), (1, 1, 200, 130, 128, "bf16"), (1, 2, 40, 70, 32, "f32"), (1, 1, 70, 33, 136, "bf16"),
    # head dims above 96 with one side on its generic-order kernel and the other on the hand-scheduled passes
    (1, 2, 40, 200, 104, "bf16"), (1, 1, 200, 40, 128, "bf16"),
])
def test_queries_and_keys_differ(B, H, M, N, d, dtype):
    """Cross-attention shapes (the paper's Background allows M != N): every element of all ten outputs against
    the oracle, for the full backward and for both one-sided ones."""
    announce(f"M != N: B{B} H{H} M{M} N{N} d{d} {dtype}")
    qs = wl.make_inputs(wl.custom(B, H, M, d, dtype), 51)   # query side: q, tq, gO, gTO
    ks = wl.make_inputs(wl.custom(B, H, N, d, dtype), 52)   # key side: k, v, tk, tv
    inp = {n: (qs if n in ("q", "tq", "gO", "gTO") else ks)[n] for n in wl.NAMES}
    dev = {n: t.cuda() for n, t in inp.items()}
    six = [dev[n] for n in wl.NAMES[:6]]
    fwd = tvm.tvmattn_jvp_fwd(*six)
    assert fwd[0].shape == (B, H, M, d) and fwd[2].shape == (B, H, M)
    grads = tvm.tvmattn_jvp_bwd(*six, *fwd, dev["gO"], dev["gTO"])
    assert grads[0].shape == (B, H, M, d) and grads[1].shape == (B, H, N, d)
    g_only = tvm.tvmattn_jvp_bwd(six[0], six[1], six[2], None, None, None, fwd[0], None, fwd[2], None, dev["gO"], None)
    t_only = tvm.tvmattn_jvp_bwd(*six, *fwd, None, dev["gTO"])
    torch.cuda.synchronize()
    tol = pu.TOL[dtype]
    for b in range(B):
        for h in range(H):
            a = [wl.to_f64(inp[n][b, h]) for n in wl.NAMES]
            ro = pu.orc.attn_jvp_fwd_head(*a[:6])
            rg = pu.orc.attn_jvp_bwd_head(*a)
            r1 = pu.orc.attn_jvp_bwd_head(*a[:6], a[6], np.zeros_like(a[6]))
            r2 = pu.orc.attn_jvp_bwd_head(*a[:6], np.zeros_like(a[6]), a[7])
            for name, got, ref in (list(zip(pu.FWD_NAMES, fwd, ro)) + list(zip(pu.BWD_NAMES, grads, rg)) +
                                   list(zip(("dq1", "dk1", "dv1"), g_only[:3], r1[:3])) +
                                   list(zip(("dq2", "dk2", "dv2", "dtq2", "dtk2", "dtv2"), t_only, r2))):
                e = pu.rel_err(got[b, h].float().cpu().numpy(), ref)
                assert e <= tol, (name, b, h, e)


def test_single_key_cross_attention():
    """One key, many queries: P = 1, so O = V and tO = tV for every query and the gradients of Q, K, tQ, tK
    vanish: on the GPU they are the rounding noise of terms that cancel (delta + Sigma_2 from the stored bf16
    o, to against DF from V, tV), bounded here against the size of those terms."""
    B, H, M, N, d = 1, 2, 129, 1, 32
    qs = wl.make_inputs(wl.custom(B, H, M, d, "bf16"), 53)
    ks = wl.make_inputs(wl.custom(B, H, N, d, "bf16"), 54)
    inp = {n: (qs if n in ("q", "tq", "gO", "gTO") else ks)[n] for n in wl.NAMES}
    dev = {n: t.cuda() for n, t in inp.items()}
    six = [dev[n] for n in wl.NAMES[:6]]
    o, to, lse, stats = tvm.tvmattn_jvp_fwd(*six)
    dq, dk, dv, dtq, dtk, dtv = tvm.tvmattn_jvp_bwd(*six, o, to, lse, stats, dev["gO"], dev["gTO"])
    torch.cuda.synchronize()
    assert torch.equal(o, dev["v"].expand(B, H, M, d))
    assert float((to.float() - dev["tv"].float()).abs().max()) <= 2e-2 * float(dev["tv"].float().abs().max())
    # sizes of the cancelling terms per query row, and of one bf16 rounding step on them
    terms = (dev["gO"].float().abs() * o.float().abs() + dev["gTO"].float().abs() * to.float().abs()).sum(dim=3).max()
    noise = float(terms) * 2.0 ** -7
    alpha = d ** -0.5
    assert float(dq.float().abs().max()) <= noise * alpha * float(dev["k"].float().abs().max())
    assert float(dtq.float().abs().max()) <= noise * alpha * float(dev["k"].float().abs().max())
    for h in range(H):
        a = [wl.to_f64(inp[n][0, h]) for n in wl.NAMES]
        ref = pu.orc.attn_jvp_bwd_head(*a)
        assert pu.rel_err(dv[0, h].float().cpu().numpy(), ref[2]) <= pu.TOL["bf16"]
        assert pu.rel_err(dtv[0, h].float().cpu().numpy(), ref[5]) <= pu.TOL["bf16"]
        # dK, dtK: sums of M such noise terms times q, tq rows
        bound = noise * alpha * M ** 0.5 * 4.0 * float(dev["q"].float().abs().max())
        assert float(dk[0, h].float().abs().max()) <= bound and float(dtk[0, h].float().abs().max()) <= bound


def test_random_shapes_against_the_oracle():
    """Forty seeded random problems (batch, heads, queries, keys, head dim, dtype, storage order of either
    side, explicit or default scale): every element of all ten outputs against the oracle."""
    import dataclasses
    rng = np.random.default_rng(2511)
    dims = [8, 16, 24, 40, 48, 64, 72, 80, 96, 104, 128, 136]
    for case in range(40):
        d = int(rng.choice(dims))
        dtype = "f32" if case % 8 == 7 else "bf16"
        B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
        # (a handful of keys is its own case: test_single_key_cross_attention and the single-token tests)
        N = int(rng.integers(8, 400)) if case % 3 else int(rng.choice([31, 32, 64, 65, 128, 129, 255, 256]))
        M = 0 if case % 2 else int(rng.integers(2, 400))
        if dtype == "f32":
            N, M = min(N, 150), min(M, 150)
        w = dataclasses.replace(wl.custom(B, H, N, d, dtype), M=M)
        scale = 0.0 if case % 4 else float(rng.uniform(0.05, 0.3))
        perm_q, perm_k = bool(rng.integers(2)), bool(rng.integers(2))
        announce(f"random case {case}: {w} scale={scale:.3f} bnhd(q side)={perm_q} bnhd(k side)={perm_k}")
        inp = wl.make_inputs(w, 1000 + case)

        def put(n, t):
            t = t.cuda()
            if perm_q if n in ("q", "tq", "gO", "gTO") else perm_k:
                t = t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
            return t
        dev = {n: put(n, t) for n, t in inp.items()}
        six = [dev[n] for n in wl.NAMES[:6]]
        fwd = tvm.tvmattn_jvp_fwd(*six, scale)
        grads = tvm.tvmattn_jvp_bwd(*six, *fwd, dev["gO"], dev["gTO"], scale)
        torch.cuda.synchronize()
        pu.check_heads(w, inp, fwd, grads, pu.all_heads(w), scale=scale or None)


def test_random_long_shapes_against_the_oracle():
    """Sixteen more seeded random problems with 400 to 1100 keys (the eight-wave forward, many tiles in every
    kernel, ragged last tiles), M = N or M drawn separately: every element of all ten outputs against the oracle."""
    import dataclasses
    rng = np.random.default_rng(19797)
    dims = [8, 24, 40, 48, 64, 72, 80, 96, 128]
    for case in range(16):
        d = int(rng.choice(dims))
        B, H = 1, int(rng.integers(1, 3))
        N = int(rng.integers(400, 1100))
        M = 0 if case % 2 else int(rng.integers(130, 1100))
        w = dataclasses.replace(wl.custom(B, H, N, d, "bf16"), M=M)
        scale = 0.0 if case % 4 else float(rng.uniform(0.05, 0.3))
        announce(f"random long case {case}: {w} scale={scale:.3f}")
        inp = wl.make_inputs(w, 3000 + case)
        fwd, grads = pu.run_gpu(inp, scale)
        pu.check_heads(w, inp, fwd, grads, pu.all_heads(w), scale=scale or None)
