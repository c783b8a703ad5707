"""tvmattn_jvp_bwd_static, the backward entry point that allocates nothing (its row vectors live in a static device
array of the library), through the C-ABI: its six outputs against tvmattn_jvp_bwd's on the same inputs, bit for bit
(same kernels, same order of every sum), on two calls in a row, the second with a smaller input, so that whatever
the first call left in the shared array is there when the second runs.  Collected last (the file name sorts behind
every other test file)."""
import ctypes
import sys

import pytest
import torch

import paper_2511_19797_amd as tvm
from paper_2511_19797_amd import binding, workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _both_ways(w, seed, flags=0):
    print(f"[case] static-scratch backward {w} flags={flags}", flush=True)
    sys.stdout.flush()
    inp = wl.make_inputs(w, seed)
    dev = {n: t.cuda() for n, t in inp.items()}
    six = [dev[n] for n in wl.NAMES[:6]]
    fwd = tvm.tvmattn_jvp_fwd(*six, flags=flags)
    ref = tvm.tvmattn_jvp_bwd(*six, *fwd, dev["gO"], dev["gTO"], flags=flags)
    # poisoned, preallocated outputs: the call under test gets nothing to allocate and must write every element
    out = tuple(torch.full_like(t, float("nan")) for t in ref)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    desc = binding.make_desc(six[1], 0.0, six[0], flags)
    ptrs = [t.data_ptr() for t in six] + [t.data_ptr() for t in fwd] + [dev["gO"].data_ptr(), dev["gTO"].data_ptr()] + \
           [t.data_ptr() for t in out]
    rc = binding.lib().tvmattn_jvp_bwd_static(ctypes.byref(desc), *ptrs[:6], ptrs[6], ptrs[7], ptrs[8], ptrs[9],
                                              ptrs[10], ptrs[11], out[0].data_ptr(), out[1].data_ptr(), out[2].data_ptr(),
                                              out[3].data_ptr(), out[4].data_ptr(), out[5].data_ptr(),
                                              ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, tvm.tvmattn_strerror(rc)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() <= before   # (the garbage collector may free earlier cases' tensors meanwhile)
    for name, a, b in zip(pu.BWD_NAMES, out, ref):
        assert torch.equal(a, b), f"{name} differs from tvmattn_jvp_bwd's"
    return inp, fwd, out


def test_static_scratch_backward_twice_second_call_smaller():
    # matrix-core path: 3 x 2 x 333 = 1998 query rows first, then 2 x 1 x 100 = 200 on the same stream
    big = wl.custom(3, 2, 333, 72, "bf16")
    small = wl.custom(2, 1, 100, 72, "bf16")
    _both_ways(big, 81)
    inp, fwd, out = _both_ways(small, 82)
    pu.check_heads(small, inp, fwd, out, pu.all_heads(small))   # and against the oracle
    # the same pair on the plain-ALU kernels (float32), whose separate row-scalar kernel writes the array
    _both_ways(wl.custom(2, 2, 150, 40, "f32"), 83)
    inp, fwd, out = _both_ways(wl.custom(1, 2, 64, 32, "f32"), 84)
    pu.check_heads(wl.custom(1, 2, 64, 32, "f32"), inp, fwd, out, [(0, 0), (0, 1)])


def test_static_scratch_backward_wide_heads_change_of_row_vector_convention():
    """Head dims above 96: the hand-scheduled passes leave the row vectors in the static array negated and in log2
    units, the generic-order kernels (64 rows or fewer on the streamed side) plain; calls of either kind in a row on
    the same array, each smaller than the one before."""
    _both_ways(wl.custom(2, 2, 200, 128, "bf16"), 87)       # passes on both sides
    _both_ways(wl.custom(1, 2, 64, 120, "bf16"), 88)        # generic-order kernels on both sides
    inp, fwd, out = _both_ways(wl.custom(1, 1, 70, 104, "bf16"), 89)   # passes again
    pu.check_heads(wl.custom(1, 1, 70, 104, "bf16"), inp, fwd, out, [(0, 0)])


def test_static_scratch_backward_m_differs_and_one_sided():
    import dataclasses
    w = dataclasses.replace(wl.custom(1, 2, 200, 64, "bf16"), M=130)
    _both_ways(w, 85)
    # one upstream gradient only, through the binding's wrapper (outputs preallocated)
    inp = wl.make_inputs(w, 86)
    dev = {n: t.cuda() for n, t in inp.items()}
    six = [dev[n] for n in wl.NAMES[:6]]
    fwd = tvm.tvmattn_jvp_fwd(*six)
    ref = tvm.tvmattn_jvp_bwd(*six, *fwd, None, dev["gTO"])
    got = tvm.tvmattn_jvp_bwd_static(*six, *fwd, None, dev["gTO"], out=tuple(torch.empty_like(t) for t in ref))
    torch.cuda.synchronize()
    for a, b in zip(got, ref):
        assert torch.equal(a, b)


def test_static_scratch_backward_at_the_headline_size():
    """C4 (262,144 query rows, a quarter of the array): bit for bit against the workspace call."""
    w = wl.CONFIGS["C4"]
    _both_ways(w, 104)
