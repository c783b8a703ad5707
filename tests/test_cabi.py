"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2511_19797_amd as tvm
from paper_2511_19797_amd import binding, build as tvm_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        tvm_build.build()
    return binding.lib()


def declared_functions():
    names = []
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if not f.endswith(".h"):
            continue
        src = open(os.path.join(inc, f)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names += re.findall(r"\b(tvmattn_\w+)\s*\(", src)
    return sorted(set(names))


def test_header_symbols_exported(L):
    names = declared_functions()
    assert {"tvmattn_jvp_fwd", "tvmattn_jvp_bwd", "tvmattn_jvp_bwd_workspace_bytes", "tvmattn_strerror",
            "tvmattn_version", "tvmattn_jvp_bwd_static", "tvmattn_jvp_bwd_timed"} <= set(names)
    for n in names:
        assert hasattr(L, n), f"{n} declared in include/ but not exported"


def test_version_and_strerror(L):
    assert tvm.tvmattn_version() >= 100
    for code in (0, -1, -2, -3, -4, -99):
        assert isinstance(tvm.tvmattn_strerror(code), str) and tvm.tvmattn_strerror(code)


def desc(B=1, H=1, N=8, D=8, dtype=1, scale=0.0, sb=0, sh=0, sn=0, M=0, flags=0, qsb=0, qsh=0, qsn=0):
    return binding.tvmattn_desc(B, H, N, D, dtype, scale, sb, sh, sn, M, flags, qsb, qsh, qsn)


def fwd_status(L, d, ptrs=None):
    p = ptrs or [0x1000000 * (i + 1) for i in range(10)]
    return L.tvmattn_jvp_fwd(ctypes.byref(d), *p, None)


@pytest.mark.parametrize("kw,status", [
    (dict(B=0), -1), (dict(N=0), -1), (dict(D=0), -1), (dict(H=-3), -1),
    (dict(D=257), -2), (dict(dtype=7), -2), (dict(scale=-1.0), -1), (dict(scale=float("nan")), -1),
    (dict(scale=float("inf")), -1),
    (dict(sn=4, sh=64, sb=64), -1),            # stride_n < D
    (dict(D=8, sn=12, sh=96, sb=96), -1),       # 24-byte row pitch is not a 16-byte multiple
    (dict(B=1 << 15, H=1 << 15, N=4), -2),      # 2^32 rows
    (dict(M=-1), -1), (dict(flags=2), -1), (dict(flags=-1), -1),
    (dict(M=16, qsn=4, qsh=64, qsb=64), -1),    # query-side row pitch < D
    (dict(M=16, qsn=12, qsh=192, qsb=192), -1), # query-side pitch not a 16-byte multiple
    (dict(B=1 << 15, H=1 << 15, N=1, M=4), -2), # 2^32 query rows
])
def test_bad_descriptors_rejected_without_gpu(L, kw, status):
    assert fwd_status(L, desc(**kw)) == status
    assert L.tvmattn_jvp_bwd_workspace_bytes(ctypes.byref(desc(**kw))) == 0


def test_null_misaligned_and_aliased_pointers(L):
    d = desc()
    good = [0x1000000 * (i + 1) for i in range(10)]
    assert L.tvmattn_jvp_fwd(None, *good, None) == -1
    for i in range(10):
        p = list(good)
        p[i] = None
        assert fwd_status(L, d, p) == -1
        p[i] = good[i] + 4
        assert fwd_status(L, d, p) == -1
    p = list(good)
    p[6] = p[0]            # o aliases q
    assert fwd_status(L, d, p) == -1
    p = list(good)
    p[7] = p[6]            # to aliases o
    assert fwd_status(L, d, p) == -1


def test_bwd_workspace_contract(L):
    d = desc(B=2, H=3, N=100, D=72)
    need = L.tvmattn_jvp_bwd_workspace_bytes(ctypes.byref(d))
    assert need >= 2 * 2 * 3 * 100 * 4 and need % 256 == 0
    ptrs = [0x1000000 * (i + 1) for i in range(19)]
    assert L.tvmattn_jvp_bwd(ctypes.byref(d), *ptrs, need - 1, None) == -3
    bad = list(ptrs)
    bad[18] = None
    assert L.tvmattn_jvp_bwd(ctypes.byref(d), *bad, need, None) == -1
    # the diagnostic flag is a per-call field of the descriptor; nothing process-wide is left
    assert not hasattr(L, "tvmattn_set_path") and not hasattr(L, "tvmattn_set_bwd_events")
    df = desc(B=2, H=3, N=100, D=72, flags=binding.TVMATTN_FLAG_PLAIN_ALU)
    assert L.tvmattn_jvp_bwd(ctypes.byref(df), *ptrs, need - 1, None) == -3
    # the timed variant: same checks, the events argument in front of the stream
    ev = (ctypes.c_void_p * 4)(None, None, None, None)
    assert L.tvmattn_jvp_bwd_timed(ctypes.byref(d), *ptrs, need - 1, ev, None) == -3
    assert L.tvmattn_jvp_bwd_timed(ctypes.byref(d), *bad, need, None, None) == -1


def test_one_sided_backward_argument_rules(L):
    """gTO NULL: the tangent tensors take no part and may be NULL too; gO NULL: everything else is
    still required; both NULL is an error.  (Status -3, workspace too small, shows that the
    pointer checks were passed; nothing is launched.)"""
    d = desc(B=2, H=3, N=100, D=72)
    need = L.tvmattn_jvp_bwd_workspace_bytes(ctypes.byref(d))
    ptrs = [0x1000000 * (i + 1) for i in range(19)]
    Q, K, V, TQ, TK, TV, O, TO, LSE, STATS, GO, GTO, DQ, DK, DV, DTQ, DTK, DTV, WS = range(19)

    def call(nulls, ws=need - 1):
        p = [None if i in nulls else x for i, x in enumerate(ptrs)]
        return L.tvmattn_jvp_bwd(ctypes.byref(d), *p, ws, None)

    assert call({GO, GTO}) == -1
    assert call({GTO}) == -3
    assert call({GTO, TQ, TK, TV, TO, STATS, DTQ, DTK, DTV}) == -3
    assert call({GTO, DQ}) == -1 and call({GTO, O}) == -1 and call({GTO, LSE}) == -1
    assert call({GO}) == -3
    assert call({GO, TQ}) == -1 and call({GO, DTK}) == -1 and call({GO, STATS}) == -1
    # forward: lse and stats are saved together or not at all (both NULL is accepted: GPU tests)
    one = [0x1000000 * (i + 1) for i in range(10)]
    one[9] = None
    assert fwd_status(L, d, one) == -1


def test_queries_and_keys_may_differ_in_number(L):
    """M queries, N keys: the workspace (one entry per query row and vector) follows M, and M = 0 means N."""
    w = lambda **kw: L.tvmattn_jvp_bwd_workspace_bytes(ctypes.byref(desc(B=2, H=3, D=16, **kw)))
    assert w(N=100) == w(N=100, M=100) == w(N=7, M=100)
    assert w(N=100, M=40) < w(N=100) < w(N=100, M=300)
    assert w(N=100, M=300) >= 3 * 2 * 3 * 300 * 4


def test_qknorm_argument_rules(L):
    """The QK-norm entry points validate before anything is launched.  (Status -3, workspace too small,
    shows that the pointer checks of the backward were passed; no call here is a valid one.)"""
    L.tvmattn_qknorm_jvp_fwd.argtypes = [ctypes.POINTER(binding.tvmattn_desc)] + [ctypes.c_void_p] * 6 + \
        [ctypes.c_float] + [ctypes.c_void_p] * 5
    L.tvmattn_qknorm_jvp_bwd.argtypes = [ctypes.POINTER(binding.tvmattn_desc)] + [ctypes.c_void_p] * 6 + \
        [ctypes.c_float] + [ctypes.c_void_p] * 11 + [ctypes.c_size_t, ctypes.c_void_p]
    L.tvmattn_qknorm_jvp_bwd_workspace_bytes.restype = ctypes.c_size_t
    d = desc(B=2, H=3, N=100, D=72, M=40)
    ins = [0x1000000 * (i + 1) for i in range(6)]
    outs = [0x1000000 * (i + 7) for i in range(4)]
    fwd = lambda i, o, eps=1e-6, dd=d: L.tvmattn_qknorm_jvp_fwd(ctypes.byref(dd), *i, eps, *o, None)
    for bad_eps in (-1.0, float("nan"), float("inf")):
        assert fwd(ins, outs, bad_eps) == -1
    assert fwd(ins, outs, dd=desc(D=0)) == -1 and fwd(ins, outs, dd=desc(dtype=9)) == -2
    for i in range(6):
        p = list(ins)
        p[i] = None
        assert fwd(p, outs) == -1
        p[i] = ins[i] + 8
        assert fwd(p, outs) == -1
    for o in range(4):
        p = list(outs)
        p[o] = None
        assert fwd(ins, p) == -1
        p[o] = ins[0]          # an output aliases q
        assert fwd(ins, p) == -1
    # backward: one partial gain-gradient row per workgroup and side, 16 rows per workgroup, at most 1024 workgroups
    need = L.tvmattn_qknorm_jvp_bwd_workspace_bytes(ctypes.byref(d))
    rows_q, rows_k = 2 * 3 * 40, 2 * 3 * 100
    assert need >= ((rows_q + 15) // 16 + (rows_k + 15) // 16) * 72 * 4 and need % 256 == 0
    big = L.tvmattn_qknorm_jvp_bwd_workspace_bytes(ctypes.byref(desc(B=64, H=16, N=1024, D=72)))
    assert big <= 2 * (1024 * 72 * 4 + 256)
    assert L.tvmattn_qknorm_jvp_bwd_workspace_bytes(ctypes.byref(desc(D=0))) == 0
    b_in = [0x1000000 * (i + 1) for i in range(6)]
    b_rest = [0x1000000 * (i + 7) for i in range(11)]   # 4 upstream gradients, 6 outputs, workspace
    bwd = lambda a, b, ws=need - 1, eps=1e-6: L.tvmattn_qknorm_jvp_bwd(ctypes.byref(d), *a, eps, *b, ws, None)
    assert bwd(b_in, b_rest) == -3
    assert bwd(b_in, b_rest, eps=-2.0) == -1
    for i in range(11):
        p = list(b_rest)
        p[i] = None
        assert bwd(b_in, p) == -1
    p = list(b_rest)
    p[5] = p[4]                # dtq aliases dq
    assert bwd(b_in, p) == -1


def test_fused_forward_argument_rules(L):
    """tvmattn_jvp_fwd_qknorm validates before anything is launched: no call here is a valid one (every pointer is
    fake), and each returns from the checks."""
    L.tvmattn_jvp_fwd_qknorm.argtypes = [ctypes.POINTER(binding.tvmattn_desc)] + [ctypes.c_void_p] * 6 + \
        [ctypes.c_float] + [ctypes.c_void_p] * 11
    d = desc(B=2, H=3, N=100, D=72, M=40)
    ins = [0x1000000 * (i + 1) for i in range(6)]          # q, tq, k, tk, gain_q, gain_k
    vs = [0x1000000 * (i + 7) for i in range(2)]           # v, tv
    outs = [0x1000000 * (i + 9) for i in range(8)]         # qn, tqn, kn, tkn, o, to, lse, stats
    call = lambda i, v, o, eps=1e-6, dd=d: L.tvmattn_jvp_fwd_qknorm(ctypes.byref(dd), *i, eps, *v, *o, None)
    for bad_eps in (-1.0, float("nan"), float("inf")):
        assert call(ins, vs, outs, bad_eps) == -1
    assert call(ins, vs, outs, dd=desc(D=0)) == -1
    # what the matrix-core forward does not take is refused, not sent elsewhere
    assert call(ins, vs, outs, dd=desc(dtype=0, D=32)) == -2 and call(ins, vs, outs, dd=desc(D=136)) == -2
    assert call(ins, vs, outs, dd=desc(D=72, flags=binding.TVMATTN_FLAG_PLAIN_ALU)) == -2
    for i in range(6):
        p = list(ins)
        p[i] = None
        assert call(p, vs, outs) == -1
        p[i] = ins[i] + 8
        assert call(p, vs, outs) == -1
    for o in range(6):
        p = list(outs)
        p[o] = None
        assert call(ins, vs, p) == -1
        p[o] = ins[0]          # an output aliases q
        assert call(ins, vs, p) == -1
    assert call(ins, vs, outs[:6] + [None, outs[7]]) == -1   # lse and stats are saved together or not at all
    assert call(ins, [None, vs[1]], outs) == -1


def test_fused_backward_argument_rules(L):
    """tvmattn_jvp_bwd_qknorm: checked before anything is launched; status -3 (workspace too small) shows that
    the pointer checks were passed, -2 that the shape is one the fused kernels do not take."""
    L.tvmattn_jvp_bwd_qknorm.argtypes = [ctypes.POINTER(binding.tvmattn_desc)] + [ctypes.c_void_p] * 6 + \
        [ctypes.c_float] + [ctypes.c_void_p] * 21 + [ctypes.c_size_t, ctypes.c_void_p]
    L.tvmattn_jvp_bwd_qknorm_workspace_bytes.restype = ctypes.c_size_t
    d = desc(B=2, H=3, N=300, D=72, M=100)
    need = L.tvmattn_jvp_bwd_qknorm_workspace_bytes(ctypes.byref(d))
    plain = L.tvmattn_jvp_bwd_workspace_bytes(ctypes.byref(d))
    assert need >= plain + (1 + 3) * 2 * 3 * 72 * 4 and need % 256 == 0   # one gain-gradient row per 128 rows of a head
    head = [0x1000000 * (i + 1) for i in range(6)]
    rest = [0x1000000 * (i + 7) for i in range(21)]   # 12 more inputs, 8 outputs, workspace
    call = lambda a, b, ws=need - 1, eps=1e-6, dd=d: L.tvmattn_jvp_bwd_qknorm(ctypes.byref(dd), *a, eps, *b, ws, None)
    assert call(head, rest) == -3
    assert call(head, rest, eps=float("nan")) == -1
    for i in range(21):
        p = list(rest)
        p[i] = None
        assert call(head, p) == -1
    p = list(rest)
    p[13] = p[12]              # dk aliases dq
    assert call(head, p) == -1
    for kw in (dict(D=128), dict(D=72, dtype=0), dict(D=20, sn=24, sh=24 * 8, sb=24 * 8)):
        dd = desc(**kw)
        assert L.tvmattn_jvp_bwd_qknorm_workspace_bytes(ctypes.byref(dd)) == 0
        assert call(head, rest, ws=1 << 30, dd=dd) == -2


def test_adaln_argument_rules(L):
    """The AdaLN modulation entry points validate before anything is launched; status -3 (workspace too small)
    shows that the backward's shape and pointer checks were passed.  The forward takes no workspace: no call of it
    here is a valid one."""
    I, P, F, Z = ctypes.c_int, ctypes.c_void_p, ctypes.c_float, ctypes.c_size_t
    L.tvmattn_adaln_jvp_fwd.argtypes = [I] * 4 + [P] * 6 + [F] + [P] * 3
    L.tvmattn_adaln_jvp_bwd.argtypes = [I] * 4 + [P] * 6 + [F] + [P] * 9 + [Z, P]
    L.tvmattn_adaln_jvp_bwd_workspace_bytes.restype, L.tvmattn_adaln_jvp_bwd_workspace_bytes.argtypes = Z, [I] * 4
    assert not hasattr(L, "tvmattn_adaln_jvp_fwd_workspace_bytes")
    B, T, C = 4, 100, 1152
    nb = L.tvmattn_adaln_jvp_bwd_workspace_bytes(B, T, C, 1)
    assert nb >= B * 4 * C * 4 and nb % 256 == 0
    for bad in ((0, T, C, 1), (B, 0, C, 1), (B, T, 0, 1), (B, T, C, 5), (B, T, 1156, 1), (B, T, 2056, 1), (B, T, 1028, 0),
                (70000, 1, 64, 1)):
        assert L.tvmattn_adaln_jvp_bwd_workspace_bytes(*bad) == 0
    ins = [0x1000000 * (i + 1) for i in range(6)]
    fouts = [0x1000000 * (i + 7) for i in range(2)]
    fwd = lambda i, o, eps=1e-6, shape=(B, T, C, 1): L.tvmattn_adaln_jvp_fwd(*shape, *i, eps, *o, None)
    assert fwd(ins, fouts, eps=-1.0) == -1 and fwd(ins, fouts, shape=(B, T, 12, 1)) == -2
    assert fwd(ins, fouts, shape=(B, T, C, 3)) == -2 and fwd(ins, fouts, shape=(B, -1, C, 1)) == -1
    for k in range(6):
        p = list(ins)
        p[k] = None
        assert fwd(p, fouts) == -1
    p = list(fouts)
    p[1] = p[0]
    assert fwd(ins, p) == -1
    assert fwd(ins, [fouts[0], ins[0] + 4096]) == -1     # ty starts inside x
    brest = [0x1000000 * (i + 7) for i in range(9)]   # gy, gty, six outputs, workspace
    bwd = lambda i, r, ws=nb - 1: L.tvmattn_adaln_jvp_bwd(B, T, C, 1, *i, 1e-6, *r, ws, None)
    assert bwd(ins, brest) == -3
    for k in range(9):
        p = list(brest)
        p[k] = None
        assert bwd(ins, p) == -1
    # the variant that adds the residual connection's gradients: both or neither, aligned, not aliased by an output
    L.tvmattn_adaln_jvp_bwd_residual.argtypes = [I] * 4 + [P] * 6 + [F] + [P] * 11 + [Z, P]
    res = lambda g, gt, r=brest, ws=nb - 1: L.tvmattn_adaln_jvp_bwd_residual(B, T, C, 1, *ins, 1e-6, r[0], r[1], g, gt, *r[2:],
                                                                          ws, None)
    assert res(None, None) == -3 and res(0x30000000, 0x31000000) == -3
    assert res(0x30000000, None) == -1 and res(None, 0x31000000) == -1 and res(0x30000004, 0x31000000) == -1
    assert res(brest[2], 0x31000000) == -1     # gx aliases gres


def test_gate_argument_rules(L):
    """The residual-gate entry points validate before anything is launched."""
    I, P, F, Z = ctypes.c_int, ctypes.c_void_p, ctypes.c_float, ctypes.c_size_t
    L.tvmattn_gate_jvp_fwd.argtypes = [I] * 4 + [P] * 6 + [F] + [P] * 3
    L.tvmattn_gate_jvp_bwd.argtypes = [I] * 4 + [P] * 4 + [F] + [P] * 7 + [Z, P]
    L.tvmattn_gate_jvp_bwd_workspace_bytes.restype, L.tvmattn_gate_jvp_bwd_workspace_bytes.argtypes = Z, [I] * 4
    B, T, C = 4, 100, 1152
    nb = L.tvmattn_gate_jvp_bwd_workspace_bytes(B, T, C, 1)
    assert nb >= B * 2 * C * 4 and nb % 256 == 0
    for bad in ((0, T, C, 1), (B, 0, C, 1), (B, T, 0, 1), (B, T, C, 5), (B, T, 1156, 1), (B, T, 2056, 1), (B, T, 1028, 0)):
        assert L.tvmattn_gate_jvp_bwd_workspace_bytes(*bad) == 0
    ins = [0x1000000 * (i + 1) for i in range(6)]
    outs = [0x1000000 * (i + 7) for i in range(2)]
    fwd = lambda i, o, eps=1e-6, shape=(B, T, C, 1): L.tvmattn_gate_jvp_fwd(*shape, *i, eps, *o, None)
    assert fwd(ins, outs, eps=-1.0) == -1 and fwd(ins, outs, shape=(B, T, 12, 1)) == -2
    assert fwd(ins, outs, shape=(B, T, C, 3)) == -2 and fwd(ins, outs, shape=(B, -1, C, 1)) == -1
    for k in range(6):
        p = list(ins)
        p[k] = None
        assert fwd(p, outs) == -1
        p[k] = ins[k] + 4     # not 16-byte aligned
        assert fwd(p, outs) == -1
    assert fwd(ins, [outs[0], outs[0]]) == -1 and fwd(ins, [ins[1], outs[1]]) == -1 and fwd(ins, [outs[0], ins[2]]) == -1
    # (z = x and tz = tx exactly are allowed: the stream updated in place; they pass the checks and would launch)
    bins = [0x1000000 * (i + 1) for i in range(4)]          # h, th, c, tc
    brest = [0x1000000 * (i + 5) for i in range(7)]         # gz, gtz, gh, gth, gc, gtc, workspace
    bwd = lambda i, r, ws=nb - 1: L.tvmattn_gate_jvp_bwd(B, T, C, 1, *i, 1e-6, *r, ws, None)
    assert bwd(bins, brest) == -3
    for k in range(7):
        p = list(brest)
        p[k] = None
        assert bwd(bins, p) == -1
    for k in range(4):
        p = list(bins)
        p[k] = None
        assert bwd(p, brest) == -1


def test_gelu_argument_rules(L):
    I, P, LL = ctypes.c_int, ctypes.c_void_p, ctypes.c_longlong
    L.tvmattn_gelu_jvp_fwd.argtypes = [LL, I] + [P] * 5
    L.tvmattn_gelu_jvp_bwd.argtypes = [LL, I] + [P] * 7
    ptr = [0x1000000 * (i + 1) for i in range(6)]
    fwd = lambda n, dt, p: L.tvmattn_gelu_jvp_fwd(n, dt, *p, None)
    bwd = lambda n, dt, p: L.tvmattn_gelu_jvp_bwd(n, dt, *p, None)
    assert fwd(0, 1, ptr[:4]) == -1 and fwd(-8, 1, ptr[:4]) == -1 and bwd(0, 1, ptr) == -1
    assert fwd(12, 1, ptr[:4]) == -2 and fwd(6, 0, ptr[:4]) == -2 and fwd(8, 7, ptr[:4]) == -2 and bwd(12, 1, ptr) == -2
    for k in range(4):
        p = list(ptr[:4])
        p[k] = None
        assert fwd(64, 1, p) == -1
        p[k] = ptr[k] + 8
        assert fwd(64, 1, p) == -1
    assert fwd(64, 1, [ptr[0], ptr[1], ptr[0], ptr[3]]) == -1 and fwd(64, 1, [ptr[0], ptr[1], ptr[2], ptr[2]]) == -1
    for k in range(6):
        p = list(ptr)
        p[k] = None
        assert bwd(64, 1, p) == -1
    assert bwd(64, 1, ptr[:4] + [ptr[4], ptr[4]]) == -1 and bwd(64, 1, ptr[:4] + [ptr[1], ptr[5]]) == -1


def test_missing_library_raises_and_nothing_falls_back(monkeypatch, tmp_path):
    """Without the built library every entry point of the binding raises: there is no CPU or eager path behind it."""
    import paper_2511_19797_amd.binding as b
    monkeypatch.setattr(b, "LIB_PATH", str(tmp_path / "libtvmattn_missing.so"))
    monkeypatch.setattr(b, "_lib", None)
    with pytest.raises(ImportError):
        b.tvmattn_version()
    with pytest.raises(ImportError):
        b.lib()
    import inspect
    src = inspect.getsource(b)
    assert "oracle" not in src, "the binding must not know the oracle"


def test_outputs_are_allocated_with_the_inputs_strides():
    """q, k, v sliced out of one fused [B,N,3,H,D] projection are not dense: the descriptor carries their strides
    and the kernels store through them, so the binding must allocate outputs with those very strides (a compact
    torch.empty_like would be overrun)."""
    import torch
    B, N, H, D = 2, 5, 4, 8
    qkv = torch.zeros(B, N, 3, H, D, dtype=torch.bfloat16)
    q = qkv[:, :, 0].permute(0, 2, 1, 3)   # [B,H,N,D] view
    assert not q.is_contiguous() and q.stride() == (N * 3 * H * D, D, 3 * H * D, 1)
    assert torch.empty_like(q).stride() != q.stride()      # what went wrong before
    o = binding._like(q)
    assert o.shape == q.shape and o.stride() == q.stride() and o.dtype == q.dtype
    d = binding.make_desc(q)
    assert (d.stride_b, d.stride_h, d.stride_n) == o.stride()[:3]
    assert (d.qstride_b, d.qstride_h, d.qstride_n) == o.stride()[:3]
    # the largest element offset the kernels can reach lies inside the allocation
    reach = sum((n - 1) * s for n, s in zip(o.shape, o.stride()))
    assert reach < o.untyped_storage().nbytes() // o.element_size()


def test_outputs_may_not_overlap_but_interleaved_slices_may(L):
    """The overlap check is exact for tensors of one layout: dq, dk, dv written as the three slices of one fused
    [B,N,3,H,D] gradient buffer interleave without sharing an element and are accepted; an output that starts inside
    an input, or a slice shifted by less than a row, is rejected.  (-3, workspace too small, = checks passed.)"""
    B, H, N, D = 2, 3, 100, 72
    sn, sh, sb = 3 * H * D, D, N * 3 * H * D          # element strides of a [B,H,N,D] view of [B,N,3,H,D]
    d = desc(B=B, H=H, N=N, D=D, sb=sb, sh=sh, sn=sn)
    need = L.tvmattn_jvp_bwd_workspace_bytes(ctypes.byref(d))
    big = 0x10000000
    bufs = [big * (i + 1) for i in range(8)]          # fused buffers: [q|k|v], [tq|tk|tv], [o|..], [to|..], [gO|..], [gTO|..], grads, tangent grads
    sl = lambda base, i: base + i * H * D * 2          # slice i of a fused buffer (bf16)
    q, k, v = (sl(bufs[0], i) for i in range(3))
    tq, tk, tv = (sl(bufs[1], i) for i in range(3))
    o, to, gO, gTO = bufs[2], bufs[3], bufs[4], bufs[5]
    lse, stats, ws = big * 9, big * 10, big * 11
    dq, dk, dv = (sl(bufs[6], i) for i in range(3))
    dtq, dtk, dtv = (sl(bufs[7], i) for i in range(3))
    call = lambda *outs: L.tvmattn_jvp_bwd(ctypes.byref(d), q, k, v, tq, tk, tv, o, to, lse, stats, gO, gTO, *outs, ws,
                                           need - 1, None)
    assert call(dq, dk, dv, dtq, dtk, dtv) == -3                       # interleaved slices: fine
    assert call(dq, dq + 16, dv, dtq, dtk, dtv) == -1                  # dk shifted by 8 elements: shares elements with dq
    assert call(dq, dk, dv, dtq, dtk, sl(bufs[0], 2) + sn * 2) == -1   # dtv = v one row down: same elements as v
    assert call(dq, dk, dv, dtq, dtk, sl(bufs[0], 1) + 32) == -1       # starts inside a row of k
    assert call(dq, dk, dv, dtq, dtk, bufs[2] + 4096) == -1            # starts inside o
    assert call(dq, dk, dv, dtq, dtk, ws) == -1                        # the workspace is an output too
    # contiguous tensors: an output that begins inside another tensor's range
    dc = desc(B=B, H=H, N=N, D=D)
    nb = B * H * N * D * 2
    ptrs = [big * (i + 1) for i in range(19)]
    needc = L.tvmattn_jvp_bwd_workspace_bytes(ctypes.byref(dc))
    assert L.tvmattn_jvp_bwd(ctypes.byref(dc), *ptrs, needc - 1, None) == -3
    p = list(ptrs)
    p[13] = p[12] + nb - 16                                             # dk starts in the last row of dq
    assert L.tvmattn_jvp_bwd(ctypes.byref(dc), *p, needc - 1, None) == -1
    p[13] = p[12] + nb                                                  # right behind it: fine
    assert L.tvmattn_jvp_bwd(ctypes.byref(dc), *p, needc - 1, None) == -3


def test_static_scratch_backward_rejects_what_does_not_fit(L):
    """tvmattn_jvp_bwd_static keeps its row vectors in a static device array of TVMATTN_STATIC_MAX_ROWS entries each:
    more query rows than that is a clear error, returned before anything touches the GPU."""
    L.tvmattn_jvp_bwd_static.argtypes = [ctypes.POINTER(binding.tvmattn_desc)] + [ctypes.c_void_p] * 19
    ptrs = [0x100000000 * (i + 1) for i in range(18)]
    too_big = desc(B=16, H=16, N=4097, D=64)          # 1,048,832 rows
    assert 16 * 16 * 4097 > binding.TVMATTN_STATIC_MAX_ROWS
    assert L.tvmattn_jvp_bwd_static(ctypes.byref(too_big), *ptrs, None) == -5
    assert "static scratch" in tvm.tvmattn_strerror(-5)
    assert L.tvmattn_jvp_bwd_static(ctypes.byref(desc(D=0)), *ptrs, None) == -1
    assert L.tvmattn_jvp_bwd_static(None, *ptrs, None) == -1
    header = open(os.path.join(ROOT, "include", "tvmattn.h")).read()
    assert re.search(r"#define\s+TVMATTN_STATIC_MAX_ROWS\s+\(1 << 20\)", header)


def test_linear_argument_rules(L):
    """The linear-layer entry points validate before anything is launched; -3 (workspace too small) shows that the
    backward's checks were passed.  No forward call here is a valid one."""
    I, P, Z, LL = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_longlong
    L.tvmattn_linear_jvp_fwd.argtypes = [I] * 4 + [P, P, LL, P, P, P, P, LL, P]
    L.tvmattn_linear_jvp_bwd.argtypes = [I] * 4 + [P, P, LL, P, P, P, LL] + [P] * 5 + [Z, P]
    L.tvmattn_linear_jvp_bwd_workspace_bytes.restype, L.tvmattn_linear_jvp_bwd_workspace_bytes.argtypes = Z, [I] * 4
    R, K, F = 1000, 1152, 3456
    need = L.tvmattn_linear_jvp_bwd_workspace_bytes(R, K, F, 1)
    assert need >= F * K * 4 + F * 4 and need % 256 == 0
    for bad in ((0, K, F, 1), (R, 0, F, 1), (R, K, -1, 1)):
        assert L.tvmattn_linear_jvp_bwd_workspace_bytes(*bad) == 0
    for unsup in ((R, K, F, 0), (R, K, F, 9), (R, 40, F, 1), (R, K, 100, 1), (R, 16, F, 1)):
        assert L.tvmattn_linear_jvp_bwd_workspace_bytes(*unsup) == 0
    G = 0x100000000
    x, tx, w, b, y, ty = (G * (i + 1) for i in range(6))
    fwd = lambda shape=(R, K, F, 1), x=x, tx=tx, w=w, b=b, y=y, ty=ty, ldx=0, ldy=0: \
        L.tvmattn_linear_jvp_fwd(*shape, x, tx, ldx, w, b, y, ty, ldy, None)
    assert fwd((0, K, F, 1)) == -1 and fwd((R, K, F, 0)) == -2 and fwd((R, 40, F, 1)) == -2
    assert fwd(x=None) == -1 and fwd(tx=None) == -1 and fwd(w=None) == -1 and fwd(y=None) == -1
    assert fwd(ty=y + 1024) == -1 and fwd(y=w + 64) == -1
    assert fwd(ldx=K - 8) == -1 and fwd(ldy=-1) == -1 and fwd(ldx=K + 4) == -2    # below K; negative; not 16-byte rows
    # x and tx as two slices of one [R, 3K] buffer (pitch 3K): they interleave without sharing an element
    assert fwd(tx=x + 2 * K, ldx=3 * K, y=x + 8) == -1                            # ... but y inside x's rows does
    gy, gty, gx, gtx, gw, gb, ws = (G * (i + 7) for i in range(7))
    bwd = lambda x=x, tx=tx, w=w, gy=gy, gty=gty, gx=gx, gtx=gtx, gw=gw, gb=gb, ws=ws, wsb=need - 1, ldx=0, ldy=0: \
        L.tvmattn_linear_jvp_bwd(R, K, F, 1, x, tx, ldx, w, gy, gty, ldy, gx, gtx, gw, gb, ws, wsb, None)
    assert bwd() == -3 and bwd(gb=None) == -3                                      # no bias gradient wanted: fine
    assert bwd(tx=x + 2 * K, gtx=gx + 2 * K, ldx=3 * K) == -3                      # slices of fused buffers
    assert bwd(tx=x + 2 * K, gtx=gx + 2 * K + 16, ldx=3 * K - 8) == -3               # (addresses are bytes: K elements in)
    assert bwd(gtx=gx + 2 * K, ldx=K) == -1                                        # dense rows: that overlaps gx
    for nul in ("x", "tx", "w", "gy", "gty", "gx", "gtx", "gw", "ws"):
        assert bwd(**{nul: None}) == -1
    assert bwd(gw=w + 4096) == -1                                                  # gw inside w
