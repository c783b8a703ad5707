#!/usr/bin/env python3
"""Benchmark of the hot path: one step = tvmattn_jvp_fwd + tvmattn_jvp_bwd over one batch of
synthetic DiT-shaped inputs resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4] [--also C3] [--no-cpu] [--ramp-ms 100] [--sweep]

value = algorithmic TFLOP/s of the whole step, 42*B*H*N^2*d flops per step (forward 12, backward
30; true head dim, no padding, no recompute counted), over exactly K timed steps.  roofline = the
kernel with the longest average launch, timed with HIP events recorded on the launch stream
around every launch of it in the timed region.  "kernels" = the per-kernel breakdown from an
untimed pass of K steps with every launch bracketed (bracketing all of them inside the timed
region would cost ~20 us per step, 10 % of a step at N = 256).  Before either pass the card is
kept under load for --ramp-ms (default 100 ms) so that both see the clock it sustains.
cpu_baseline = the float64 oracle timed on this machine's host cores on a bounded sample of heads of
the same workload.  Side sections, all outside the timed region and each timed after half of
--ramp-ms of the same call: one_sided (one upstream gradient alone; the forward that saves nothing),
graph_replay (the step captured in a HIP graph), qknorm, adaln, gate, gelu (the block's memory-bound
pieces, priced against 8 TB/s), linear (the block's four linear layers with tangents, against the matrix-core peak),
block (one whole block, forward and backward, as a chain of library calls), peaks (the card's own matrix-core and HBM rates from plain microbenchmarks).
roofline.traffic comes from the committed counter summary under profiles/ and is null once the kernel's sources
differ from the ones that were profiled.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "fwd+JVP and bwd attention TFLOP/s & %MFMA peak at DiT-XL/2 N=256/1024"
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
NOMINAL_MHZ = 2400.0        # the shader clock that figure is quoted at (256 CUs x 4 SIMDs x 1024 flop per cycle)
PEAK_HBM_GBS = 8000.0

# Algorithmic flops per launch, in units of B*H*N^2*d.  The six score-type products of the
# backward are counted once, with the key-side kernel; the query-side kernel's recompute of
# them is overhead, not algorithmic work.  12 + 24 + 6 = 42.
KERNEL_FLOP_UNITS = {"fwd": 12.0, "bwd_pre": 0.0, "bwd_col": 24.0, "bwd_row": 6.0}

# HBM traffic per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (KiB per dispatch), each scaled by what the
# same counter reads for a 256 MiB copy (FETCH_SIZE x2.0, WRITE_SIZE x1.0).  The figures are not kept here: they are
# read from the table rows "| traffic | <workload> | <kernel> | <FETCH KiB> | <WRITE KiB> | <source hash> |" of
# profiles/tvmattn_kernels_C4_counters.md, and a row counts only while the hash recorded with it equals the hash of
# the kernel's sources as they are now (a kernel that changed since it was profiled reports traffic = null).
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "tvmattn_kernels_C4_counters.md")
FETCH_FACTOR, WRITE_FACTOR = 2.0, 1.0
_CSRC = os.path.join(ROOT, "paper_2511_19797_amd", "csrc")
KERNEL_SOURCES = {
    "fwd": ("fwd_mfma.hip", "mfma_tiles.h", "tvm_common.h"),
    "bwd_row": ("bwd_row_pipe.hip", "pipe_ops.h", "mfma_tiles.h", "tvm_common.h"),
    "bwd_col": ("bwd_col_pipe.hip", "pipe_ops.h", "mfma_tiles.h", "tvm_common.h"),
}


def source_sha16(kernel):
    import hashlib
    h = hashlib.sha256()
    for f in KERNEL_SOURCES[kernel]:
        with open(os.path.join(_CSRC, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(workload, kernel):
    """Bytes per launch from the committed counter summary, or None (no row, or the kernel's sources changed)."""
    import re
    if kernel not in KERNEL_SOURCES or not os.path.exists(TRAFFIC_PROFILE):
        return None
    pat = re.compile(r"^\|\s*traffic\s*\|\s*(\w+)\s*\|\s*(\w+)\s*\|\s*([\d.]+)\s*\|\s*([\d.]+)\s*\|\s*([0-9a-f]{16})\s*\|")
    with open(TRAFFIC_PROFILE) as fh:
        for line in fh:
            m = pat.match(line)
            if m and m.group(1) == workload and m.group(2) == kernel:
                if m.group(5) != source_sha16(kernel):
                    return None
                return float(m.group(3)) * 1024.0 * FETCH_FACTOR + float(m.group(4)) * 1024.0 * WRITE_FACTOR
    return None


# Backward latency of the paper's own kernels on one H100 (App. C "Evaluation"; batch size and head
# dim not stated there), by (H, S): context for --sweep, whose batch 1 / head dim 64 are our choice.
PAPER_H100_BWD_MS = {
    (1, 128): 1.31, (1, 1024): 1.38, (1, 4096): 1.96, (1, 8192): 3.98, (1, 16384): 10.06, (1, 32768): 40.24,
    (24, 128): 1.40, (24, 1024): 1.42, (24, 4096): 15.13, (24, 8192): 58.70, (24, 16384): 238.4, (24, 32768): 958.6,
}


class Hip:
    """The handful of HIP runtime calls needed for event timing on torch's stream."""

    def __init__(self):
        self.rt = ctypes.CDLL("libamdhip64.so")
        self.rt.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.rt.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.rt.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.rt.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.rt.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def check(self, rc, what):
        if rc != 0:
            raise RuntimeError(f"{what} failed with hipError {rc}")

    def event(self):
        e = ctypes.c_void_p()
        self.check(self.rt.hipEventCreate(ctypes.byref(e)), "hipEventCreate")
        return e.value

    def record(self, e, stream):
        self.check(self.rt.hipEventRecord(e, stream), "hipEventRecord")

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        self.check(self.rt.hipEventSynchronize(b), "hipEventSynchronize")
        self.check(self.rt.hipEventElapsedTime(ctypes.byref(ms), a, b), "hipEventElapsedTime")
        return float(ms.value)

    def destroy(self, e):
        self.rt.hipEventDestroy(e)


RAMP_MS = 100.0  # untimed load before any measurement; see run_workload


def run_workload(w, steps, warmup, hip, seed=2024, ramp_ms=RAMP_MS):
    import torch

    import paper_2511_19797_amd as tvm
    from paper_2511_19797_amd import workloads as wl

    inp = wl.make_inputs(w, seed)
    dev = {n: t.cuda() for n, t in inp.items()}
    del inp
    six = [dev[n] for n in wl.NAMES[:6]]
    B, H, N, d, M = w.B, w.H, w.N, w.d, w.Mq
    fwd_out = (torch.empty_like(six[0]), torch.empty_like(six[0]),
               torch.empty((B, H, M), dtype=torch.float32, device="cuda"),
               torch.empty((B, H, M), dtype=torch.float32, device="cuda"))
    bwd_out = tuple(torch.empty_like(six[0] if n in (0, 3) else six[1]) for n in range(6))  # dq, dk, dv, dtq, dtk, dtv
    ws = torch.empty(tvm.tvmattn_jvp_bwd_workspace_bytes(six[0], k=six[1]), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream

    def step(ev=None):
        """ev: None, or six handles; a zero handle skips that record."""
        if ev is not None and ev[0]:
            hip.record(ev[0], stream)
        tvm.tvmattn_jvp_fwd(*six, out=fwd_out)
        if ev is not None:
            if ev[1]:
                hip.record(ev[1], stream)
        tvm.tvmattn_jvp_bwd(*six, *fwd_out, dev["gO"], dev["gTO"], out=bwd_out, workspace=ws,
                            events=None if ev is None else ev[2:6])

    names = ("fwd", "bwd_pre", "bwd_col", "bwd_row")
    pairs = ((0, 1), (2, 3), (4, 5), (3, 4))  # bwd events: start, after pre, after row, after col

    for _ in range(warmup):
        step()
    # The card needs 30-40 ms of continuous load to reach the clock it then sustains (measured: the
    # first 10 steps of C4 after an idle second take 1.30 ms each, steps 40 to 2000 1.08 ms), and
    # allocating the next workload's inputs is idle time enough to lose it: keep stepping, untimed,
    # until `ramp_ms` of load have gone by.
    torch.cuda.synchronize()
    t_ramp = time.perf_counter()
    while (time.perf_counter() - t_ramp) * 1e3 < ramp_ms:
        for _ in range(8):
            step()
        torch.cuda.synchronize()
    # Untimed pass with every launch bracketed: the per-kernel breakdown, and which kernel dominates.
    # (Event records between the launches cost ~20 us per step, which matters at N = 256.)
    events = [[hip.event() for _ in range(6)] for _ in range(steps)]
    for k in range(steps):
        step(events[k])
    torch.cuda.synchronize()
    kern_ms = {n: sum(hip.elapsed_ms(ev[a], ev[b]) for ev in events) / steps for n, (a, b) in zip(names, pairs)}
    dominant = max(names, key=lambda n: kern_ms[n])
    # The timed region: exactly `steps` steps, only the dominant kernel bracketed by events.
    a, b = dict(zip(names, pairs))[dominant]
    timed = [[(ev[i] if i in (a, b) else 0) for i in range(6)] for ev in events]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        step(timed[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dom_ms = sum(hip.elapsed_ms(ev[a], ev[b]) for ev in events) / steps
    for ev in events:
        for e in ev:
            hip.destroy(e)
    for t in list(fwd_out) + list(bwd_out):
        assert bool(torch.isfinite(t.float()).all()), "non-finite output in the timed region"

    unit = float(B) * H * M * N * d
    ms_step = (t1 - t0) * 1e3 / steps
    res = {
        "workload": f"{w.name} {w.note}: B={B} H={H} N={N} d={d} {w.dtype}" + (f" M={M}" if M != N else ""),
        "ms_per_step": ms_step,
        "tflops": 42.0 * unit / (ms_step * 1e-3) / 1e12,
        "kernels": {},
    }
    for n in names:
        ms = kern_ms[n]
        fl = KERNEL_FLOP_UNITS[n] * unit
        res["kernels"][n] = {"ms": ms, "tflops": fl / (ms * 1e-3) / 1e12 if ms > 0 else None}
    res["fwd_tflops"] = res["kernels"]["fwd"]["tflops"]
    bwd_ms = kern_ms["bwd_pre"] + kern_ms["bwd_col"] + kern_ms["bwd_row"]
    res["bwd_tflops"] = 30.0 * unit / (bwd_ms * 1e-3) / 1e12
    res["fwd_hbm_gbs"] = w.fwd_bytes() / (kern_ms["fwd"] * 1e-3) / 1e9
    res["bwd_hbm_gbs"] = w.bwd_bytes() / (bwd_ms * 1e-3) / 1e9
    res["dominant"] = {"kernel": dominant, "ms_in_timed_region": dom_ms}
    return res, kern_ms, unit


def one_sided(w, steps, seed=2024):
    """Backward with one upstream gradient only, and the forward that saves nothing, timed outside
    the timed region of the headline figure (wall clock over `steps` calls each after a short ramp, device
    synchronised)."""
    import torch

    import paper_2511_19797_amd as tvm
    from paper_2511_19797_amd import workloads as wl

    inp = wl.make_inputs(w, seed)
    dev = {n: t.cuda() for n, t in inp.items()}
    del inp
    q, k, v, tq, tk, tv = [dev[n] for n in wl.NAMES[:6]]
    fwd_out = tvm.tvmattn_jvp_fwd(q, k, v, tq, tk, tv)
    o, to, lse, stats = fwd_out
    nosave = (torch.empty_like(o), torch.empty_like(o), None, None)
    g6 = tuple(torch.empty_like(q if n in (0, 3) else k) for n in range(6))  # dq, dk, dv, dtq, dtk, dtv
    g3 = g6[:3] + (None, None, None)
    ws = torch.empty(tvm.tvmattn_jvp_bwd_workspace_bytes(q, k=k), dtype=torch.uint8, device="cuda")
    unit = float(w.B) * w.H * w.Mq * w.N * w.d
    cases = {
        # the ordinary attention backward: 5 of the 15 products (S, G V^T, and three output products)
        "bwd_gO_only": (10.0, lambda: tvm.tvmattn_jvp_bwd(q, k, v, None, None, None, o, None, lse, None, dev["gO"], None,
                                                          out=g3, workspace=ws)),
        # the tangent path alone: 13 of the 15
        "bwd_gTO_only": (26.0, lambda: tvm.tvmattn_jvp_bwd(q, k, v, tq, tk, tv, o, to, lse, stats, None, dev["gTO"],
                                                           out=g6, workspace=ws)),
        "fwd_nothing_saved": (12.0, lambda: tvm.tvmattn_jvp_fwd(q, k, v, tq, tk, tv, out=nosave, save=False)),
    }
    out = {}
    for name, (units, fn) in cases.items():
        ms = _timed_ms(fn, steps)
        out[name] = {"ms": ms, "tflops": units * unit / (ms * 1e-3) / 1e12}
    return out


def graph_step(w, steps, ramp_ms=100.0, seed=2024):
    """One forward + backward step captured in a HIP graph (the library allocates nothing, issues no memset and never
    synchronises, so it can be captured as it is) and replayed `steps` times: what a training loop that captures
    its step pays per step, without the caller's per-call overhead.  Wall clock per replay."""
    import torch

    import paper_2511_19797_amd as tvm
    from paper_2511_19797_amd import workloads as wl

    dev = {n: t.cuda() for n, t in wl.make_inputs(w, seed).items()}
    six = [dev[n] for n in wl.NAMES[:6]]
    fo = tvm.tvmattn_jvp_fwd(*six)
    go = tvm.tvmattn_jvp_bwd(*six, *fo, dev["gO"], dev["gTO"])
    ws = torch.empty(max(tvm.tvmattn_jvp_bwd_workspace_bytes(six[0], k=six[1]), 16), dtype=torch.uint8, device="cuda")

    def step():
        tvm.tvmattn_jvp_fwd(*six, out=fo)
        tvm.tvmattn_jvp_bwd(*six, *fo, dev["gO"], dev["gTO"], out=go, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    t0, ramp = time.perf_counter(), 0  # the same 100 ms under load as the eager measurement gets (the clock ramps up)
    while time.perf_counter() - t0 < ramp_ms * 1e-3:
        graph.replay()
        torch.cuda.synchronize()
        ramp += 1
    ms = _timed_ms(graph.replay, steps)
    # launches: every step this function ran, eager or replayed (2 eager, the ramp, 3 warm-up replays, the timed ones)
    return {"ms_per_step": ms, "launches": 2 + ramp + 3 + steps, "tflops": 42.0 * w.B * w.H * w.Mq * w.N * w.d / (ms * 1e-3) / 1e12}


def _marker():
    """One tiny float32 forward (the plain-ALU kernel, which nothing else in a default run launches) right behind the
    headline's timed region: in a kernel trace, the launches of the step's kernels just before it are that region."""
    import torch

    import paper_2511_19797_amd as tvm

    t = [torch.zeros(1, 1, 8, 8, device="cuda") for _ in range(6)]
    tvm.tvmattn_jvp_fwd(*t)
    torch.cuda.synchronize()


SIDE_RAMP_MS = 50.0  # load before a side measurement (half of --ramp-ms): the sections start from an idle device, i.e. a low clock


def _timed_ms(fn, steps):
    """Wall clock per call over `steps` calls, after SIDE_RAMP_MS of the same call (at least 3 of them), device
    synchronised on both sides."""
    import torch

    t0, n = time.perf_counter(), 0
    while n < 3 or (time.perf_counter() - t0) * 1e3 < SIDE_RAMP_MS:
        fn()
        n += 1
        if n % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def _sclk_under(fn, secs=1.6):
    """Shader clock in MHz as rocm-smi reports it about a second into a load: `fn` (one asynchronous call) is kept
    running for `secs` seconds while a thread asks rocm-smi once.  None where rocm-smi is missing or says nothing
    that parses.  (The card holds its nominal 2400 MHz under a copy and under bare matrix-core instructions, and
    settles lower under kernels that also keep LDS, VALU and HBM busy: what they could reach at most scales with it.)"""
    import re
    import subprocess
    import threading

    import torch

    got = []

    def ask():
        time.sleep(0.7)
        try:
            r = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=10)
            m = re.search(r"sclk clock level:\s*\d+:\s*\((\d+)Mhz\)", r.stdout)
            if m:
                got.append(int(m.group(1)))
        except Exception:
            pass

    th = threading.Thread(target=ask)
    th.start()
    t0, n = time.perf_counter(), 0
    while time.perf_counter() - t0 < secs or th.is_alive():
        fn()
        n += 1
        if n % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    th.join()
    return got[0] if got else None


def sustained_clock(w, seed=2024):
    """The shader clock under the workload's own step (forward + backward back to back)."""
    import torch

    import paper_2511_19797_amd as tvm
    from paper_2511_19797_amd import workloads as wl

    dev = {n: t.cuda() for n, t in wl.make_inputs(w, seed).items()}
    six = [dev[n] for n in wl.NAMES[:6]]
    fo = tvm.tvmattn_jvp_fwd(*six)
    go = tvm.tvmattn_jvp_bwd(*six, *fo, dev["gO"], dev["gTO"])
    ws = torch.empty(max(tvm.tvmattn_jvp_bwd_workspace_bytes(six[0], k=six[1]), 16), dtype=torch.uint8, device="cuda")

    def step():
        tvm.tvmattn_jvp_fwd(*six, out=fo)
        tvm.tvmattn_jvp_bwd(*six, *fo, dev["gO"], dev["gTO"], out=go, workspace=ws)
    return _sclk_under(step)


def _hbm_cases(cases, steps):
    """cases: name -> (algorithmic bytes per call, callable).  Times each and prices it against 8 TB/s."""
    out = {}
    for name, (nbytes, fn) in cases.items():
        ms = _timed_ms(fn, steps)
        gbs = nbytes / (ms * 1e-3) / 1e9
        out[name] = {"ms": ms, "algorithmic_bytes": nbytes, "GBps": gbs, "bound": "hbm", "peak": 8000.0,
                     "frac": gbs / 8000.0}
    return out


def qknorm(w, steps, seed=2024):
    """The QK-norm with tangent that feeds the attention (RMSNorm with gain, Sec. "Semi-Lipschitz control"),
    forward and backward on the workload's q and k, timed outside the timed region of the headline figure
    (wall clock over `steps` calls each, device synchronised).  Memory-bound: algorithmic bytes = every
    tensor once (forward reads 4 and writes 4, backward reads 8 and writes 4), against 8 TB/s."""
    import torch

    import paper_2511_19797_amd as tvm
    from paper_2511_19797_amd import workloads as wl

    inp = wl.make_inputs(w, seed)
    dev = {n: inp[n].cuda() for n in ("q", "tq", "k", "tk", "gO", "gTO", "v", "tv")}
    del inp
    gq, gk = [g.cuda() for g in wl.make_gains(w, seed + 1)]
    q, tq, k, tk = dev["q"], dev["tq"], dev["k"], dev["tk"]
    fo = tuple(torch.empty_like(t) for t in (q, q, k, k))
    bo = tuple(torch.empty_like(t) for t in (q, q, k, k)) + (torch.empty_like(gq), torch.empty_like(gk))
    ws = torch.empty(tvm.tvmattn_qknorm_jvp_bwd_workspace_bytes(q, k=k), dtype=torch.uint8, device="cuda")
    side_bytes = float(w.B) * w.H * w.d * (2 if w.dtype == "bf16" else 4)
    tensors_q, tensors_k = side_bytes * w.Mq, side_bytes * w.N
    cases = {
        "fwd": (4.0 * (tensors_q + tensors_k),
                lambda: tvm.tvmattn_qknorm_jvp_fwd(q, tq, k, tk, gq, gk, 1e-6, out=fo)),
        # upstream gradients: any tensors of the right shapes
        "bwd": (6.0 * (tensors_q + tensors_k),
                lambda: tvm.tvmattn_qknorm_jvp_bwd(q, tq, k, tk, gq, gk, 1e-6, dev["gO"], dev["gTO"], dev["v"], dev["tv"],
                                                   out=bo, workspace=ws)),
    }
    timed = lambda fn: _timed_ms(fn, steps)
    out = _hbm_cases(cases, steps)
    # the block as the paper runs it: attention on the normalised tensors, then both backwards, as two calls and
    # as the one call that does the norm's backward in the attention kernels' epilogues (where that is served)
    if tvm.tvmattn_jvp_bwd_qknorm_workspace_bytes(q, k=k) > 0:
        qn, tqn, kn, tkn = tvm.tvmattn_qknorm_jvp_fwd(q, tq, k, tk, gq, gk, 1e-6, out=fo)
        v, tv, gO, gTO = dev["v"], dev["tv"], dev["gO"], dev["gTO"]
        o, to, lse, stats = tvm.tvmattn_jvp_fwd(qn, kn, v, tqn, tkn, tv)
        g6 = tuple(torch.empty_like(q if n in (0, 3) else k) for n in range(6))
        aws = torch.empty(tvm.tvmattn_jvp_bwd_workspace_bytes(q, k=k), dtype=torch.uint8, device="cuda")
        fws = torch.empty(tvm.tvmattn_jvp_bwd_qknorm_workspace_bytes(q, k=k), dtype=torch.uint8, device="cuda")
        f8 = tuple(torch.empty_like(t) for t in g6) + (torch.empty_like(gq), torch.empty_like(gk))

        def two_calls():
            tvm.tvmattn_jvp_bwd(qn, kn, v, tqn, tkn, tv, o, to, lse, stats, gO, gTO, out=g6, workspace=aws)
            tvm.tvmattn_qknorm_jvp_bwd(q, tq, k, tk, gq, gk, 1e-6, g6[0], g6[3], g6[1], g6[4], out=bo, workspace=ws)

        out["attention_bwd_then_norm_bwd"] = {"ms": timed(two_calls)}
        out["attention_bwd_with_norm_bwd_fused"] = {"ms": timed(lambda: tvm.tvmattn_jvp_bwd_qknorm(
            q, tq, k, tk, gq, gk, 1e-6, qn, tqn, kn, tkn, v, tv, o, to, lse, stats, gO, gTO, out=f8, workspace=fws))}
    # the forward likewise: norm then attention as two calls, and as the one call that normalises the query side
    # where the attention kernel loads its query rows (where the matrix-core forward is served)
    if w.dtype == "bf16" and w.d % 8 == 0 and w.d <= 128:
        v, tv = dev["v"], dev["tv"]
        rows = lambda: torch.empty((w.B, w.H, w.Mq), dtype=torch.float32, device="cuda")
        f4 = (torch.empty_like(q), torch.empty_like(q), rows(), rows())
        f8b = tuple(torch.empty_like(t) for t in (q, q, k, k, q, q)) + (rows(), rows())

        def two_fwd_calls():
            n4 = tvm.tvmattn_qknorm_jvp_fwd(q, tq, k, tk, gq, gk, 1e-6, out=fo)
            tvm.tvmattn_jvp_fwd(n4[0], n4[2], v, n4[1], n4[3], tv, out=f4)

        out["norm_fwd_then_attention_fwd"] = {"ms": timed(two_fwd_calls)}
        out["attention_fwd_with_query_norm_fused"] = {"ms": timed(lambda: tvm.tvmattn_jvp_fwd_qknorm(
            q, tq, k, tk, gq, gk, 1e-6, v, tv, out=f8b))}
    return out


def adaln(w, steps, seed=2024):
    """The normalised AdaLN modulation with tangent (Sec. "Semi-Lipschitz control"; the operand of ATTN and MLP in
    the paper's block) at the workload's token count and hidden size H*d, forward and backward, timed outside the
    timed region of the headline figure.  Memory-bound: algorithmic bytes = every [B,T,C] tensor once (forward
    reads 2 and writes 2, backward reads 4 and writes 2), against 8 TB/s."""
    import torch

    import paper_2511_19797_amd as tvm
    from paper_2511_19797_amd import workloads as wl

    B, T, C = w.B, w.Mq, w.H * w.d
    inp = wl.make_adaln_inputs(B, T, C, w.dtype, seed)
    dev = {n: t.cuda() for n, t in inp.items()}
    del inp
    args = [dev[n] for n in ("x", "tx", "a", "ta", "b", "tb")]
    fo = (torch.empty_like(dev["x"]), torch.empty_like(dev["x"]))
    bo = fo + tuple(torch.empty_like(dev["a"]) for _ in range(4))
    ws = torch.empty(1 << 26, dtype=torch.uint8, device="cuda")
    one = float(B) * T * C * (2 if w.dtype == "bf16" else 4)
    cases = {"fwd": (4.0 * one, lambda: tvm.tvmattn_adaln_jvp_fwd(*args, 1e-6, out=fo)),
             "bwd": (6.0 * one, lambda: tvm.tvmattn_adaln_jvp_bwd(*args, 1e-6, dev["gy"], dev["gty"], out=bo, workspace=ws))}
    out = {"shape": {"B": B, "T": T, "C": C}}
    out.update(_hbm_cases(cases, steps))
    return out


def gate(w, steps, seed=2024):
    """The normalised gate of a residual branch with tangent (App. "Full Description of Normalization of Modulation":
    how the output of ATTN and of MLP re-enters the stream) at the workload's token count and hidden size H*d,
    forward and backward, timed outside the timed region of the headline figure.  Memory-bound: algorithmic bytes =
    every [B,T,C] tensor once (forward reads 4 and writes 2, backward reads 4 and writes 2), against 8 TB/s."""
    import torch

    import paper_2511_19797_amd as tvm
    from paper_2511_19797_amd import workloads as wl

    B, T, C = w.B, w.Mq, w.H * w.d
    inp = wl.make_gate_inputs(B, T, C, w.dtype, seed)
    dev = {n: t.cuda() for n, t in inp.items()}
    del inp
    fo = (torch.empty_like(dev["x"]), torch.empty_like(dev["x"]))
    bo = fo + (torch.empty_like(dev["c"]), torch.empty_like(dev["c"]))
    ws = torch.empty(1 << 26, dtype=torch.uint8, device="cuda")
    one = float(B) * T * C * (2 if w.dtype == "bf16" else 4)
    cases = {"fwd": (6.0 * one, lambda: tvm.tvmattn_gate_jvp_fwd(dev["x"], dev["tx"], dev["h"], dev["th"], dev["c"],
                                                               dev["tc"], 1e-6, out=fo)),
             "bwd": (6.0 * one, lambda: tvm.tvmattn_gate_jvp_bwd(dev["h"], dev["th"], dev["c"], dev["tc"], 1e-6,
                                                               dev["gz"], dev["gtz"], out=bo, workspace=ws))}
    out = {"shape": {"B": B, "T": T, "C": C}}
    out.update(_hbm_cases(cases, steps))
    return out


def gelu(w, steps, seed=2024):
    """The MLP's activation with tangent (tanh-form GELU; the hidden layer is 4 x the model width) at the workload's
    token count, forward and backward.  Memory-bound: algorithmic bytes = every tensor once (forward reads 2 and
    writes 2, backward reads 4 and writes 2), against 8 TB/s."""
    import torch

    import paper_2511_19797_amd as tvm
    from paper_2511_19797_amd import workloads as wl

    shape = (w.B, w.Mq, 4 * w.H * w.d)
    dev = {n: t.cuda() for n, t in wl.make_gelu_inputs(shape, w.dtype, seed).items()}
    fo = (torch.empty_like(dev["u"]), torch.empty_like(dev["u"]))
    one = float(dev["u"].numel()) * dev["u"].element_size()
    cases = {"fwd": (4.0 * one, lambda: tvm.tvmattn_gelu_jvp_fwd(dev["u"], dev["tu"], out=fo)),
             "bwd": (6.0 * one, lambda: tvm.tvmattn_gelu_jvp_bwd(dev["u"], dev["tu"], dev["ga"], dev["gta"], out=fo))}
    out = {"shape": list(shape)}
    out.update(_hbm_cases(cases, steps))
    return out


def linear(w, steps, seed=2024):
    """The four linear layers of the block (fused q, k, v projection, output projection, the MLP's two; App. "Full
    Description of Normalization of Modulation") on the workload's B x M tokens at hidden size H*d, each with tangent:
    forward (one product over the stacked rows [x; tx]: 4 R K F flops) and backward (grad x over the stacked rows and
    grad W over both row sets: 8 R K F flops), priced against the bf16 matrix-core peak."""
    import torch

    import paper_2511_19797_amd as tvm
    from paper_2511_19797_amd import workloads as wl

    R, C = w.B * w.Mq, w.H * w.d
    out = {"tokens": R}
    for name, K, F in (("qkv", C, 3 * C), ("proj", C, C), ("mlp_up", C, 4 * C), ("mlp_down", 4 * C, C)):
        d = {n: t.cuda() for n, t in wl.make_linear_inputs(R, K, F, w.dtype, seed).items()}
        fo = (torch.empty(R, F, dtype=d["x"].dtype, device="cuda"), torch.empty(R, F, dtype=d["x"].dtype, device="cuda"))
        bo = (torch.empty_like(d["x"]), torch.empty_like(d["x"]), torch.empty_like(d["w"]), torch.empty_like(d["b"]))
        ws = torch.empty(tvm.tvmattn_linear_jvp_bwd_workspace_bytes(d["x"], d["w"]), dtype=torch.uint8, device="cuda")
        fms = _timed_ms(lambda: tvm.tvmattn_linear_jvp_fwd(d["x"], d["tx"], d["w"], d["b"], out=fo), steps)
        bms = _timed_ms(lambda: tvm.tvmattn_linear_jvp_bwd(d["x"], d["tx"], d["w"], d["gy"], d["gty"], out=bo, workspace=ws), steps)
        fl = 4.0 * R * K * F
        out[name] = {"K": K, "F": F, "fwd_ms": fms, "fwd_tflops": fl / (fms * 1e-3) / 1e12, "bwd_ms": bms,
                     "bwd_tflops": 2.0 * fl / (bms * 1e-3) / 1e12, "bound": "mfma", "peak": PEAK_BF16_TFLOPS,
                     "fwd_frac": fl / (fms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                     "bwd_frac": 2.0 * fl / (bms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
        del d, fo, bo, ws
    return out


def block_step(w, steps, seed=2024):
    """One whole normalised DiT block with tangent (modulation, fused projection, QK-norm, attention, projection, gate,
    modulation, MLP, gate), forward and backward, as the chain of library calls in paper_2511_19797_amd/block.py at the
    workload's batch, tokens and heads.  Wall clock per forward + backward (the chain allocates its intermediates through
    torch's caching allocator: what a training step pays)."""
    import torch

    from paper_2511_19797_amd import block, workloads as wl

    x, tx, mods, tmods, params, gz, gtz = wl.make_block_inputs(w.B, w.Mq, w.H, w.d, 4 * w.H * w.d, seed)
    dev = lambda t: t.cuda()
    x, tx, gz, gtz = dev(x), dev(tx), dev(gz), dev(gtz)
    dm, dtm, dp = ({k: dev(v) for k, v in m.items()} for m in (mods, tmods, params))

    def step():
        z, tz, saved = block.block_jvp_fwd(x, tx, dm, dtm, dp, w.H, 1e-6, 1e-6)
        block.block_jvp_bwd(x, tx, dm, dtm, dp, w.H, 1e-6, 1e-6, saved, gz, gtz)
    ms = _timed_ms(step, max(3, steps // 2))
    # the same chain captured in a HIP graph and replayed (about 50 launches per step: what the gaps between them cost)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    ms_graph = _timed_ms(graph.replay, max(3, steps // 2))
    R, C = w.B * w.Mq, w.H * w.d
    gemm = 12.0 * R * C * (3 * C + C + 4 * C + 4 * C)          # the four layers, forward 4 R K F + backward 8 R K F
    attn = 42.0 * w.B * w.H * w.Mq * w.N * w.d
    return {"ms_fwd_bwd": ms, "algorithmic_tflops": (gemm + attn) / (ms * 1e-3) / 1e12,
            "ms_fwd_bwd_graph_replay": ms_graph, "flops": {"linear_layers": gemm, "attention": attn}}


def peaks(steps):
    """The card's own ceilings, measured beside the kernels: the rate of the matrix-core instruction the attention
    kernels use (two waves per SIMD issuing it back to back) and the HBM rate of a plain copy and a plain read of
    1 GiB, each after SIDE_RAMP_MS of the same load.  The roofline's `peak` stays the published figure; these say
    how much of it this card sustains."""
    import torch

    from paper_2511_19797_amd import build as b
    if not os.path.exists(b.PEAKS_LIB):
        raise ImportError(f"{b.PEAKS_LIB} not found: run __graft_entry__.build() first")
    L = ctypes.CDLL(b.PEAKS_LIB)
    L.tvmpeaks_mfma_bf16.restype = ctypes.c_double
    L.tvmpeaks_mfma_bf16.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    L.tvmpeaks_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
    L.tvmpeaks_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    stream = torch.cuda.current_stream().cuda_stream
    blocks = 2 * torch.cuda.get_device_properties(0).multi_processor_count   # two waves per SIMD
    out = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    iters = 4000   # 64,000 products per wave, about 1 ms
    flops = []

    def mfma():
        flops.append(L.tvmpeaks_mfma_bf16(blocks, iters, out.data_ptr(), stream))
    ms = _timed_ms(mfma, steps)
    assert flops[-1] > 0, "matrix-core rate kernel failed to launch"
    res = {"mfma_bf16_tflops": flops[-1] / (ms * 1e-3) / 1e12, "mfma_ms": ms,
           "mfma_note": "v_mfma_f32_32x32x16_bf16, 4 independent accumulators per wave, 2 waves per SIMD"}
    if SIDE_RAMP_MS > 0:
        res["mfma_sclk_mhz"] = _sclk_under(mfma)
    # the same stream of products on operands that differ from product to product and from lane to lane (pseudo-random
    # in [-1, 1)): same products per cycle, but the matrix cores draw more power and the card lowers its clock
    L.tvmpeaks_mfma_bf16_random.restype = ctypes.c_double
    L.tvmpeaks_mfma_bf16_random.argtypes = L.tvmpeaks_mfma_bf16.argtypes

    def mfma_random():
        flops.append(L.tvmpeaks_mfma_bf16_random(blocks, iters, out.data_ptr(), stream))
    ms = _timed_ms(mfma_random, steps)
    assert flops[-1] > 0, "matrix-core rate kernel (random operands) failed to launch"
    res["mfma_bf16_tflops_random_operands"] = flops[-1] / (ms * 1e-3) / 1e12
    if SIDE_RAMP_MS > 0:
        res["mfma_random_operands_sclk_mhz"] = _sclk_under(mfma_random)
    # ... and with 8 of the 32 rows of one operand live, the rest zero (the last output block of a head dim of 72)
    L.tvmpeaks_mfma_bf16_random_padded.restype = ctypes.c_double
    L.tvmpeaks_mfma_bf16_random_padded.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]

    def mfma_padded():
        flops.append(L.tvmpeaks_mfma_bf16_random_padded(blocks, iters, 8, out.data_ptr(), stream))
    ms = _timed_ms(mfma_padded, steps)
    assert flops[-1] > 0, "matrix-core rate kernel (padded operands) failed to launch"
    res["mfma_bf16_tflops_issued_with_8_of_32_rows_live"] = flops[-1] / (ms * 1e-3) / 1e12
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    flag = torch.zeros(4, dtype=torch.int32, device="cuda")
    wg = 16 * torch.cuda.get_device_properties(0).multi_processor_count
    ms = _timed_ms(lambda: L.tvmpeaks_copy(dst.data_ptr(), src.data_ptr(), n, wg, stream), steps)
    res["copy_gbs"] = 2.0 * n / (ms * 1e-3) / 1e9   # bytes read + bytes written
    ms = _timed_ms(lambda: L.tvmpeaks_read(src.data_ptr(), n, flag.data_ptr(), wg, stream), steps)
    res["read_gbs"] = n / (ms * 1e-3) / 1e9
    assert torch.equal(src[:1 << 20], dst[:1 << 20]) and torch.equal(src[-(1 << 20):], dst[-(1 << 20):])
    del src, dst
    # float32 atomic adds into L2-resident per-head tiles, in the pattern and volume a backward that formed dQ, dtQ in
    # its key-side pass would need at C4 (256 heads x 8 workgroups x 4 waves, each adding 2 x 1024 x 72 floats per pass
    # over the queries: 4.8 GB per backward; reduced across the four waves of a workgroup first it would be 1.2 GB)
    L.tvmpeaks_atomic_add.restype = ctypes.c_double
    L.tvmpeaks_atomic_add.argtypes = [ctypes.c_void_p] + [ctypes.c_int] * 6 + [ctypes.c_void_p]
    heads, per_head, rows, cols = 256, 8, 1024, 72
    acc = torch.zeros(heads * 2 * rows * cols, dtype=torch.float32, device="cuda")
    nbytes = []
    ms4 = _timed_ms(lambda: nbytes.append(L.tvmpeaks_atomic_add(acc.data_ptr(), heads, per_head, rows, cols, 1, 4, stream)), steps)
    assert nbytes[-1] > 0
    res["atomic_add_f32_gbs"] = nbytes[-1] / (ms4 * 1e-3) / 1e9
    ms1 = _timed_ms(lambda: nbytes.append(L.tvmpeaks_atomic_add(acc.data_ptr(), heads, per_head, rows, cols, 1, 1, stream)), steps)
    res["atomic_add_ms_for_a_C4_backward"] = {"every_wave_adds": ms4, "one_wave_per_workgroup_adds": ms1}
    return res


def cpu_baseline(w, budget_s=20.0, seed=2024):
    """Times the oracle (forward + backward, whole heads) until about `budget_s` seconds are spent."""
    from oracle import tvmattn_oracle as orc
    from paper_2511_19797_amd import workloads as wl

    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    small = wl.custom(1, min(w.heads, 256), w.N, w.d, w.dtype, w.tangent_std, w.key_scale)
    inp = wl.make_inputs(small, seed)
    arrs = [wl.to_f64(inp[n]) for n in wl.NAMES]
    done, t0 = 0, time.perf_counter()
    while done < small.H:
        a = [x[0, done] for x in arrs]
        orc.attn_jvp_fwd_head(*a[:6])
        orc.attn_jvp_bwd_head(*a)
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    flops = 42.0 * done * w.Mq * w.N * w.d
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{done} of {w.heads} heads of {w.name} (N={w.N}, d={w.d}), float64 numpy, "
                      f"forward+backward, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--ramp-ms", type=float, default=RAMP_MS,
                    help="untimed stepping after the warm-up steps until the clock has ramped (0: none)")
    ap.add_argument("--workload", default="C4")
    ap.add_argument("--also", default="C2,C3,C5", help="comma-separated extra workloads reported under 'also'")
    ap.add_argument("--source-hashes", action="store_true",
                    help="print the hashes of the kernels' sources (what a traffic row of the counter summary records) and exit")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--sweep", action="store_true",
                    help="also time the shapes of the paper's kernel benchmark (H in 1, 24; S = 128 ... 32768) under 'sweep'")
    args = ap.parse_args()
    if args.source_hashes:
        print(json.dumps({k: source_sha16(k) for k in KERNEL_SOURCES}))
        return
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X); --gpus must be 1. "
              "Heads shard over GPUs with no exchange; no multi-GPU figure is produced.", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2511_19797_amd import workloads as wl
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    hip = Hip()
    w = wl.CONFIGS[args.workload]
    global SIDE_RAMP_MS
    SIDE_RAMP_MS = 0.5 * args.ramp_ms  # (--ramp-ms 0: counter runs, a handful of launches per kernel)
    res, kern_ms, unit = run_workload(w, args.steps, args.warmup, hip, ramp_ms=args.ramp_ms)
    _marker()

    dom = res["dominant"]["kernel"]
    dom_ms = res["dominant"]["ms_in_timed_region"]  # HIP events around every launch of it in the timed region
    achieved = KERNEL_FLOP_UNITS[dom] * unit / (dom_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_BF16_TFLOPS, "avg_launch_ms": dom_ms,
                "traffic": measured_traffic(w.name, dom)}

    also = {}
    for name in [x for x in args.also.split(",") if x and x != args.workload]:
        r, _, _ = run_workload(wl.CONFIGS[name], args.steps, args.warmup, hip, ramp_ms=args.ramp_ms)
        also[name] = r

    out = {
        "metric": METRIC, "value": res["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": res["workload"], "flops_per_step": 42.0 * unit,
                   "flop_formula": "42*B*H*M*N*d with M = N queries (fwd 12, bwd 30)"},
        "pct_mfma_peak": 100.0 * res["tflops"] / PEAK_BF16_TFLOPS,
        "fwd_tflops": res["fwd_tflops"], "bwd_tflops": res["bwd_tflops"],
        "fwd_hbm_gbs": res["fwd_hbm_gbs"], "bwd_hbm_gbs": res["bwd_hbm_gbs"],
        "kernels": res["kernels"], "roofline": roofline, "also": also,
    }
    out["one_sided"] = one_sided(w, args.steps)
    out["graph_replay"] = {name: graph_step(wl.CONFIGS[name], args.steps, args.ramp_ms) for name in dict.fromkeys([w.name] + list(also))
                           if name in wl.CONFIGS}
    out["qknorm"] = qknorm(w, args.steps)
    if w.dtype == "bf16" and (w.H * w.d) % 8 == 0 and w.H * w.d <= 2048:
        out["adaln"] = adaln(w, args.steps)
        out["gate"] = gate(w, args.steps)
        out["gelu"] = gelu(w, args.steps)
        if (w.H * w.d) % 32 == 0:
            out["linear"] = linear(w, args.steps)
            out["block"] = block_step(w, args.steps)
    if args.sweep:
        out["sweep"] = []
        for sw in wl.sweep_configs():
            # a few steps suffice for the long sequences (a step at H = 24, S = 32768 takes ~0.1 s)
            k = max(3, min(args.steps, int(2e14 / (42.0 * sw.B * sw.H * sw.N * sw.N * sw.d))))
            r, km, _ = run_workload(sw, k, min(args.warmup, k), hip, ramp_ms=args.ramp_ms)
            out["sweep"].append({
                "H": sw.H, "S": sw.N, "B": sw.B, "d": sw.d, "steps": k, "ms_per_step": r["ms_per_step"],
                "fwd_ms": km["fwd"], "bwd_ms": km["bwd_pre"] + km["bwd_row"] + km["bwd_col"], "tflops": r["tflops"],
                "paper_h100_bwd_ms": PAPER_H100_BWD_MS.get((sw.H, sw.N))})
    out["peaks"] = peaks(args.steps)
    out["roofline"]["frac_of_measured_mfma_rate"] = achieved / out["peaks"]["mfma_bf16_tflops"]
    out["roofline"]["frac_of_measured_mfma_rate_random_operands"] = achieved / out["peaks"]["mfma_bf16_tflops_random_operands"]
    if args.ramp_ms > 0:  # (not in counter runs, which keep to a handful of launches per kernel)
        mhz = sustained_clock(w)
        out["clock"] = {"nominal_mhz": NOMINAL_MHZ, "sclk_mhz_under_the_step": mhz,
                        "sclk_mhz_under_the_mfma_microbenchmark": out["peaks"].get("mfma_sclk_mhz"),
                        "sclk_mhz_under_the_mfma_microbenchmark_random_operands": out["peaks"].get("mfma_random_operands_sclk_mhz")}
        if mhz:  # the published peak is quoted at the nominal clock: what the same units give at the clock this load runs at
            out["roofline"]["frac_at_the_clock_under_load"] = achieved / (PEAK_BF16_TFLOPS * mhz / NOMINAL_MHZ)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
