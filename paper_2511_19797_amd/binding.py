"""ctypes binding of libtvmattn.so: argument marshalling only.

Same names as the C entry points (include/tvmattn.h).  torch supplies device
memory and the current stream; every step of the computation runs in the
library's HIP kernels.  There is no fallback: if the shared library is missing
or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtvmattn.so")

TVMATTN_F32, TVMATTN_BF16 = 0, 1
TVMATTN_FLAG_PLAIN_ALU = 1
TVMATTN_STATIC_MAX_ROWS = 1 << 20


class tvmattn_desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("N", ctypes.c_int32), ("D", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("scale", ctypes.c_float),
                ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64),
                ("M", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("qstride_b", ctypes.c_int64), ("qstride_h", ctypes.c_int64), ("qstride_n", ctypes.c_int64)]


class TvmattnError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"tvmattn status {status}: {msg}")
        self.status = status


_lib = None
_P = ctypes.c_void_p


def lib():
    """Loads the library on first use; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: run `python -m paper_2511_19797_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        L.tvmattn_version.restype = ctypes.c_int
        L.tvmattn_strerror.restype = ctypes.c_char_p
        L.tvmattn_strerror.argtypes = [ctypes.c_int]
        L.tvmattn_jvp_fwd.restype = ctypes.c_int
        L.tvmattn_jvp_fwd.argtypes = [ctypes.POINTER(tvmattn_desc)] + [_P] * 11
        L.tvmattn_jvp_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.tvmattn_jvp_bwd_workspace_bytes.argtypes = [ctypes.POINTER(tvmattn_desc)]
        L.tvmattn_jvp_bwd.restype = ctypes.c_int
        L.tvmattn_jvp_bwd.argtypes = [ctypes.POINTER(tvmattn_desc)] + [_P] * 19 + [ctypes.c_size_t, _P]
        L.tvmattn_jvp_bwd_timed.restype = ctypes.c_int
        L.tvmattn_jvp_bwd_timed.argtypes = ([ctypes.POINTER(tvmattn_desc)] + [_P] * 19 +
                                            [ctypes.c_size_t, ctypes.POINTER(_P), _P])
        L.tvmattn_jvp_bwd_static.restype = ctypes.c_int
        L.tvmattn_jvp_bwd_static.argtypes = [ctypes.POINTER(tvmattn_desc)] + [_P] * 19
        L.tvmattn_qknorm_jvp_fwd.restype = ctypes.c_int
        L.tvmattn_qknorm_jvp_fwd.argtypes = [ctypes.POINTER(tvmattn_desc)] + [_P] * 6 + [ctypes.c_float] + [_P] * 5
        L.tvmattn_jvp_fwd_qknorm.restype = ctypes.c_int
        L.tvmattn_jvp_fwd_qknorm.argtypes = [ctypes.POINTER(tvmattn_desc)] + [_P] * 6 + [ctypes.c_float] + [_P] * 11
        L.tvmattn_qknorm_jvp_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.tvmattn_qknorm_jvp_bwd_workspace_bytes.argtypes = [ctypes.POINTER(tvmattn_desc)]
        L.tvmattn_qknorm_jvp_bwd.restype = ctypes.c_int
        L.tvmattn_qknorm_jvp_bwd.argtypes = ([ctypes.POINTER(tvmattn_desc)] + [_P] * 6 + [ctypes.c_float] + [_P] * 11 +
                                             [ctypes.c_size_t, _P])
        L.tvmattn_jvp_bwd_qknorm_workspace_bytes.restype = ctypes.c_size_t
        L.tvmattn_jvp_bwd_qknorm_workspace_bytes.argtypes = [ctypes.POINTER(tvmattn_desc)]
        L.tvmattn_jvp_bwd_qknorm.restype = ctypes.c_int
        L.tvmattn_jvp_bwd_qknorm.argtypes = ([ctypes.POINTER(tvmattn_desc)] + [_P] * 6 + [ctypes.c_float] + [_P] * 21 +
                                             [ctypes.c_size_t, _P])
        _I = ctypes.c_int
        L.tvmattn_adaln_jvp_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.tvmattn_adaln_jvp_bwd_workspace_bytes.argtypes = [_I] * 4
        L.tvmattn_adaln_jvp_fwd.restype = ctypes.c_int
        L.tvmattn_adaln_jvp_fwd.argtypes = [_I] * 4 + [_P] * 6 + [ctypes.c_float] + [_P] * 3
        L.tvmattn_adaln_jvp_bwd.restype = ctypes.c_int
        L.tvmattn_adaln_jvp_bwd.argtypes = [_I] * 4 + [_P] * 6 + [ctypes.c_float] + [_P] * 9 + [ctypes.c_size_t, _P]
        L.tvmattn_adaln_jvp_bwd_residual.restype = ctypes.c_int
        L.tvmattn_adaln_jvp_bwd_residual.argtypes = [_I] * 4 + [_P] * 6 + [ctypes.c_float] + [_P] * 11 + [ctypes.c_size_t, _P]
        L.tvmattn_gelu_jvp_fwd.restype = ctypes.c_int
        L.tvmattn_gelu_jvp_fwd.argtypes = [ctypes.c_longlong, _I] + [_P] * 5
        L.tvmattn_gelu_jvp_bwd.restype = ctypes.c_int
        L.tvmattn_gelu_jvp_bwd.argtypes = [ctypes.c_longlong, _I] + [_P] * 7
        L.tvmattn_gate_jvp_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.tvmattn_gate_jvp_bwd_workspace_bytes.argtypes = [_I] * 4
        L.tvmattn_gate_jvp_fwd.restype = ctypes.c_int
        L.tvmattn_gate_jvp_fwd.argtypes = [_I] * 4 + [_P] * 6 + [ctypes.c_float] + [_P] * 3
        L.tvmattn_gate_jvp_bwd.restype = ctypes.c_int
        L.tvmattn_gate_jvp_bwd.argtypes = [_I] * 4 + [_P] * 4 + [ctypes.c_float] + [_P] * 7 + [ctypes.c_size_t, _P]
        L.tvmattn_linear_jvp_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.tvmattn_linear_jvp_bwd_workspace_bytes.argtypes = [_I] * 4
        L.tvmattn_linear_jvp_fwd.restype = ctypes.c_int
        _LL = ctypes.c_longlong
        L.tvmattn_linear_jvp_fwd.argtypes = [_I] * 4 + [_P, _P, _LL, _P, _P, _P, _P, _LL, _P]
        L.tvmattn_linear_jvp_bwd.restype = ctypes.c_int
        L.tvmattn_linear_jvp_bwd.argtypes = [_I] * 4 + [_P, _P, _LL, _P, _P, _P, _LL] + [_P] * 5 + [ctypes.c_size_t, _P]
        _lib = L
    return _lib


def tvmattn_version():
    return lib().tvmattn_version()


def tvmattn_strerror(status):
    return lib().tvmattn_strerror(int(status)).decode()


def _check(status):
    if status != 0:
        raise TvmattnError(status, tvmattn_strerror(status))


def make_desc(x: torch.Tensor, scale=0.0, q: torch.Tensor = None, flags=0) -> tvmattn_desc:
    """Descriptor for key-side tensors shaped and strided like `x` [B,H,N,D] and query-side tensors like `q`
    [B,H,M,D] (default: like `x`); any strides with unit innermost stride.  `flags`: TVMATTN_FLAG_* bits."""
    q = x if q is None else q
    for t in (x, q):
        if t.dim() != 4:
            raise ValueError("expected [B,H,N,D] tensors")
        if t.stride(3) != 1:
            raise ValueError("innermost stride must be 1")
    if x.dtype == torch.float32:
        dt = TVMATTN_F32
    elif x.dtype == torch.bfloat16:
        dt = TVMATTN_BF16
    else:
        raise ValueError(f"unsupported dtype {x.dtype}")
    B, H, N, D = x.shape
    if q.dtype != x.dtype or (q.shape[0], q.shape[1], q.shape[3]) != (B, H, D):
        raise ValueError("query-side and key-side tensors must agree in B, H, D and dtype")
    return tvmattn_desc(B, H, N, D, dt, float(scale), x.stride(0), x.stride(1), x.stride(2),
                        q.shape[2], int(flags), q.stride(0), q.stride(1), q.stride(2))


def _same_layout(ref, *ts):
    for t in ts:
        if t.shape != ref.shape or t.stride() != ref.stride() or t.dtype != ref.dtype or t.device != ref.device:
            raise ValueError("all tensors of one side (query side [B,H,M,D], key side [B,H,N,D]) of a call must "
                             "share shape, strides, dtype and device")
        if not t.is_cuda:
            raise ValueError("device tensors required")


def _like(ref):
    """A new tensor with exactly `ref`'s shape AND strides.  The descriptor carries one set of strides per side, taken
    from the inputs, and every kernel store uses them; torch.empty_like keeps strides only for dense tensors (a q
    sliced out of a fused [B,N,3,H,D] projection would get a compact output that the kernels then overrun)."""
    return torch.empty_strided(ref.shape, ref.stride(), dtype=ref.dtype, device=ref.device)


def _stream():
    return _P(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return None if t is None else t.data_ptr()


def tvmattn_jvp_fwd(q, k, v, tq, tk, tv, scale=0.0, out=None, save=True, flags=0):
    """Returns (o, to, lse, stats).  `out`, if given, is that same tuple of preallocated tensors.
    save=False: nothing is kept for a backward (lse and stats are None)."""
    _same_layout(q, tq)
    _same_layout(k, v, tk, tv)
    desc = make_desc(k, scale, q, flags)
    B, H, N, _ = q.shape  # row vectors go with the queries
    if out is None:
        o, to = _like(q), _like(q)
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device) if save else None
        stats = torch.empty((B, H, N), dtype=torch.float32, device=q.device) if save else None
    else:
        o, to, lse, stats = out
        _same_layout(q, o, to)
    _check(lib().tvmattn_jvp_fwd(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(), tq.data_ptr(),
                                 tk.data_ptr(), tv.data_ptr(), o.data_ptr(), to.data_ptr(), _ptr(lse), _ptr(stats),
                                 _stream()))
    return o, to, lse, stats


def tvmattn_jvp_bwd_workspace_bytes(q, scale=0.0, k=None):
    """`q`: a query-side tensor; `k`: a key-side one (default: self-attention, shaped like `q`)."""
    desc = make_desc(q if k is None else k, scale, q)
    return int(lib().tvmattn_jvp_bwd_workspace_bytes(ctypes.byref(desc)))


def _bwd_args(q, k, v, tq, tk, tv, o, to, lse, stats, gO, gTO, scale, out, flags):
    _same_layout(*[t for t in (q, tq, o, to, gO, gTO) if t is not None])
    _same_layout(*[t for t in (k, v, tk, tv) if t is not None])
    desc = make_desc(k, scale, q, flags)
    if out is None:  # dq, dk, dv, dtq, dtk, dtv
        out = tuple(_like(q if n in (0, 3) else k) if (gTO is not None or n < 3) else None for n in range(6))
    else:
        _same_layout(q, *[t for n, t in enumerate(out) if t is not None and n in (0, 3)])
        _same_layout(k, *[t for n, t in enumerate(out) if t is not None and n not in (0, 3)])
    dq, dk, dv, dtq, dtk, dtv = out
    ptrs = [q.data_ptr(), k.data_ptr(), v.data_ptr(), _ptr(tq), _ptr(tk), _ptr(tv), o.data_ptr(), _ptr(to),
            lse.data_ptr(), _ptr(stats), _ptr(gO), _ptr(gTO), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), _ptr(dtq),
            _ptr(dtk), _ptr(dtv)]
    return desc, out, ptrs


def tvmattn_jvp_bwd(q, k, v, tq, tk, tv, o, to, lse, stats, gO, gTO, scale=0.0, out=None, workspace=None, flags=0,
                    events=None):
    """Returns (dq, dk, dv, dtq, dtk, dtv).

    gTO=None: the ordinary attention backward (gradient of <gO, O> alone); tq, tk, tv, to, stats may be
    None and dtq, dtk, dtv come back as None.  gO=None: the gradient of <gTO, tO> alone.
    events: None, or four raw hipEvent_t handles (ints, created with timing enabled; None or 0 skips that
    record): the call goes through tvmattn_jvp_bwd_timed."""
    desc, out, ptrs = _bwd_args(q, k, v, tq, tk, tv, o, to, lse, stats, gO, gTO, scale, out, flags)
    need = int(lib().tvmattn_jvp_bwd_workspace_bytes(ctypes.byref(desc)))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    wsb = workspace.numel() * workspace.element_size()
    if events is None:
        _check(lib().tvmattn_jvp_bwd(ctypes.byref(desc), *ptrs, workspace.data_ptr(), wsb, _stream()))
    else:
        arr = (_P * 4)(*[_P(int(e)) if e else _P(None) for e in events])
        _check(lib().tvmattn_jvp_bwd_timed(ctypes.byref(desc), *ptrs, workspace.data_ptr(), wsb, arr, _stream()))
    return out


def tvmattn_jvp_bwd_static(q, k, v, tq, tk, tv, o, to, lse, stats, gO, gTO, scale=0.0, out=None, flags=0):
    """tvmattn_jvp_bwd without a workspace: the library's static device scratch holds the row vectors (at most
    TVMATTN_STATIC_MAX_ROWS query rows B*H*M).  The entry point itself allocates nothing; pass `out` to keep this
    wrapper from allocating the six gradients."""
    desc, out, ptrs = _bwd_args(q, k, v, tq, tk, tv, o, to, lse, stats, gO, gTO, scale, out, flags)
    _check(lib().tvmattn_jvp_bwd_static(ctypes.byref(desc), *ptrs, _stream()))
    return out


def _gain_ok(g, ref):
    if g.dtype != torch.float32 or g.dim() != 1 or g.shape[0] != ref.shape[3] or not g.is_contiguous() or g.device != ref.device:
        raise ValueError("gains must be contiguous float32 [D] tensors on the inputs' device")


def tvmattn_qknorm_jvp_fwd(q, tq, k, tk, gain_q, gain_k, eps, out=None):
    """Returns (qn, tqn, kn, tkn): RMSNorm with gain of the rows of q and k, and the tangents along tq, tk."""
    _same_layout(q, tq)
    _same_layout(k, tk)
    _gain_ok(gain_q, q)
    _gain_ok(gain_k, k)
    desc = make_desc(k, 0.0, q)
    if out is None:
        out = (_like(q), _like(q), _like(k), _like(k))
    else:
        _same_layout(q, out[0], out[1])
        _same_layout(k, out[2], out[3])
    _check(lib().tvmattn_qknorm_jvp_fwd(ctypes.byref(desc), q.data_ptr(), tq.data_ptr(), k.data_ptr(), tk.data_ptr(),
                                        gain_q.data_ptr(), gain_k.data_ptr(), float(eps), out[0].data_ptr(),
                                        out[1].data_ptr(), out[2].data_ptr(), out[3].data_ptr(), _stream()))
    return out


def tvmattn_jvp_fwd_qknorm(q, tq, k, tk, gain_q, gain_k, eps, v, tv, scale=0.0, out=None, save=True):
    """The QK-norm and the attention forward in one call (the query side is normalised inside the attention kernel).
    Returns (qn, tqn, kn, tkn, o, to, lse, stats); `out`, if given, is that tuple of preallocated tensors.
    Raises TvmattnError (unsupported) for what the matrix-core forward does not take: make the two calls there."""
    _same_layout(q, tq)
    _same_layout(k, tk, v, tv)
    _gain_ok(gain_q, q)
    _gain_ok(gain_k, k)
    desc = make_desc(k, scale, q)
    B, H, M, _ = q.shape
    if out is None:
        rows = lambda: torch.empty((B, H, M), dtype=torch.float32, device=q.device) if save else None
        out = (_like(q), _like(q), _like(k), _like(k), _like(q), _like(q), rows(), rows())
    else:
        _same_layout(q, out[0], out[1], out[4], out[5])
        _same_layout(k, out[2], out[3])
    _check(lib().tvmattn_jvp_fwd_qknorm(ctypes.byref(desc), q.data_ptr(), tq.data_ptr(), k.data_ptr(), tk.data_ptr(),
                                        gain_q.data_ptr(), gain_k.data_ptr(), float(eps), v.data_ptr(), tv.data_ptr(),
                                        out[0].data_ptr(), out[1].data_ptr(), out[2].data_ptr(), out[3].data_ptr(),
                                        out[4].data_ptr(), out[5].data_ptr(), _ptr(out[6]), _ptr(out[7]), _stream()))
    return out


def tvmattn_qknorm_jvp_bwd_workspace_bytes(q, k=None):
    desc = make_desc(q if k is None else k, 0.0, q)
    return int(lib().tvmattn_qknorm_jvp_bwd_workspace_bytes(ctypes.byref(desc)))


def tvmattn_qknorm_jvp_bwd(q, tq, k, tk, gain_q, gain_k, eps, gqn, gtqn, gkn, gtkn, out=None, workspace=None):
    """Returns (dq, dtq, dk, dtk, dgain_q, dgain_k)."""
    _same_layout(q, tq, gqn, gtqn)
    _same_layout(k, tk, gkn, gtkn)
    _gain_ok(gain_q, q)
    _gain_ok(gain_k, k)
    desc = make_desc(k, 0.0, q)
    if out is None:
        out = (_like(q), _like(q), _like(k), _like(k), torch.empty_like(gain_q), torch.empty_like(gain_k))
    else:
        _same_layout(q, out[0], out[1])
        _same_layout(k, out[2], out[3])
        _gain_ok(out[4], q)
        _gain_ok(out[5], k)
    need = int(lib().tvmattn_qknorm_jvp_bwd_workspace_bytes(ctypes.byref(desc)))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    _check(lib().tvmattn_qknorm_jvp_bwd(ctypes.byref(desc), q.data_ptr(), tq.data_ptr(), k.data_ptr(), tk.data_ptr(),
                                        gain_q.data_ptr(), gain_k.data_ptr(), float(eps), gqn.data_ptr(), gtqn.data_ptr(),
                                        gkn.data_ptr(), gtkn.data_ptr(), *[t.data_ptr() for t in out],
                                        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream()))
    return out


def tvmattn_jvp_bwd_qknorm_workspace_bytes(q, k=None):
    """0 where the fused call is not supported (see tvmattn_jvp_bwd_qknorm)."""
    desc = make_desc(q if k is None else k, 0.0, q)
    return int(lib().tvmattn_jvp_bwd_qknorm_workspace_bytes(ctypes.byref(desc)))


def tvmattn_jvp_bwd_qknorm(q, tq, k, tk, gain_q, gain_k, eps, qn, tqn, kn, tkn, v, tv, o, to, lse, stats, gO, gTO,
                           scale=0.0, out=None, workspace=None):
    """Attention backward and QK-norm backward in one call.  Returns (dq, dk, dv, dtq, dtk, dtv, dgain_q, dgain_k),
    the first six with respect to the tensors before the normalisation.  Raises TvmattnError (status -2) for
    shapes the fused kernels do not take."""
    _same_layout(q, tq, qn, tqn, o, to, gO, gTO)
    _same_layout(k, tk, kn, tkn, v, tv)
    _gain_ok(gain_q, q)
    _gain_ok(gain_k, k)
    desc = make_desc(k, scale, q)
    if out is None:
        out = tuple(_like(q if n in (0, 3) else k) for n in range(6)) + (torch.empty_like(gain_q), torch.empty_like(gain_k))
    else:
        _same_layout(q, out[0], out[3])
        _same_layout(k, out[1], out[2], out[4], out[5])
        _gain_ok(out[6], q)
        _gain_ok(out[7], k)
    need = int(lib().tvmattn_jvp_bwd_qknorm_workspace_bytes(ctypes.byref(desc)))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    _check(lib().tvmattn_jvp_bwd_qknorm(ctypes.byref(desc), q.data_ptr(), tq.data_ptr(), k.data_ptr(), tk.data_ptr(),
                                        gain_q.data_ptr(), gain_k.data_ptr(), float(eps), qn.data_ptr(), tqn.data_ptr(),
                                        kn.data_ptr(), tkn.data_ptr(), v.data_ptr(), tv.data_ptr(), o.data_ptr(),
                                        to.data_ptr(), lse.data_ptr(), stats.data_ptr(), gO.data_ptr(), gTO.data_ptr(),
                                        *[t.data_ptr() for t in out], workspace.data_ptr(),
                                        workspace.numel() * workspace.element_size(), _stream()))
    return out


def _adaln_args(x, tx, mods):
    if x.dim() != 3 or not x.is_contiguous() or not x.is_cuda:
        raise ValueError("expected contiguous [B,T,C] device tensors")
    if tx.shape != x.shape or tx.dtype != x.dtype or not tx.is_contiguous():
        raise ValueError("x and its tangent must agree in shape, dtype and layout")
    B, T, C = x.shape
    for m in mods:
        if m.shape != (B, C) or m.dtype != torch.float32 or not m.is_contiguous() or m.device != x.device:
            raise ValueError("scale, shift and their tangents must be contiguous float32 [B,C] tensors")
    dt = TVMATTN_F32 if x.dtype == torch.float32 else TVMATTN_BF16 if x.dtype == torch.bfloat16 else None
    if dt is None:
        raise ValueError(f"unsupported dtype {x.dtype}")
    return B, T, C, dt


def tvmattn_adaln_jvp_fwd(x, tx, a, ta, b, tb, eps, out=None):
    """Returns (y, ty): RMSNorm^-(x) * RMSNorm^-(a) + RMSNorm^-(b) and its tangent along (tx, ta, tb)."""
    B, T, C, dt = _adaln_args(x, tx, (a, ta, b, tb))
    y, ty = out if out is not None else (torch.empty_like(x), torch.empty_like(x))
    _check(lib().tvmattn_adaln_jvp_fwd(B, T, C, dt, x.data_ptr(), tx.data_ptr(), a.data_ptr(), ta.data_ptr(), b.data_ptr(),
                                       tb.data_ptr(), float(eps), y.data_ptr(), ty.data_ptr(), _stream()))
    return y, ty


def tvmattn_adaln_jvp_bwd(x, tx, a, ta, b, tb, eps, gy, gty, out=None, workspace=None, gres=None, gtres=None):
    """Returns (gx, gtx, ga, gta, gb, gtb).  gres, gtres (both or neither): gradients that reach x and tx along the
    residual connection, added to gx and gtx (tvmattn_adaln_jvp_bwd_residual)."""
    B, T, C, dt = _adaln_args(x, tx, (a, ta, b, tb))
    _adaln_args(gy, gty, ())
    if gy.shape != x.shape or gy.dtype != x.dtype:
        raise ValueError("upstream gradients must look like x")
    if (gres is None) != (gtres is None):
        raise ValueError("gres and gtres come together")
    if gres is not None:
        _adaln_args(gres, gtres, ())
        if gres.shape != x.shape or gres.dtype != x.dtype:
            raise ValueError("residual gradients must look like x")
    if out is None:
        out = (torch.empty_like(x), torch.empty_like(x)) + tuple(torch.empty_like(a) for _ in range(4))
    need = int(lib().tvmattn_adaln_jvp_bwd_workspace_bytes(B, T, C, dt))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    _check(lib().tvmattn_adaln_jvp_bwd_residual(B, T, C, dt, x.data_ptr(), tx.data_ptr(), a.data_ptr(), ta.data_ptr(),
                                                b.data_ptr(), tb.data_ptr(), float(eps), gy.data_ptr(), gty.data_ptr(),
                                                gres.data_ptr() if gres is not None else None,
                                                gtres.data_ptr() if gtres is not None else None,
                                                *[t.data_ptr() for t in out], workspace.data_ptr(), workspace.numel(),
                                                _stream()))
    return out


def tvmattn_gate_jvp_fwd(x, tx, h, th, c, tc, eps, out=None):
    """Returns (z, tz): x + RMSNorm^-(c) * h and its tangent along (tx, th, tc)."""
    B, T, C, dt = _adaln_args(x, tx, (c, tc))
    _adaln_args(h, th, ())
    if h.shape != x.shape or h.dtype != x.dtype:
        raise ValueError("the branch output must look like x")
    z, tz = out if out is not None else (torch.empty_like(x), torch.empty_like(x))
    _check(lib().tvmattn_gate_jvp_fwd(B, T, C, dt, x.data_ptr(), tx.data_ptr(), h.data_ptr(), th.data_ptr(), c.data_ptr(),
                                      tc.data_ptr(), float(eps), z.data_ptr(), tz.data_ptr(), _stream()))
    return z, tz


def tvmattn_gate_jvp_bwd(h, th, c, tc, eps, gz, gtz, out=None, workspace=None):
    """Returns (gh, gth, gc, gtc); the gradients with respect to x and tx are gz and gtz themselves."""
    B, T, C, dt = _adaln_args(h, th, (c, tc))
    _adaln_args(gz, gtz, ())
    if gz.shape != h.shape or gz.dtype != h.dtype:
        raise ValueError("upstream gradients must look like h")
    if out is None:
        out = (torch.empty_like(h), torch.empty_like(h), torch.empty_like(c), torch.empty_like(c))
    need = int(lib().tvmattn_gate_jvp_bwd_workspace_bytes(B, T, C, dt))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=h.device)
    _check(lib().tvmattn_gate_jvp_bwd(B, T, C, dt, h.data_ptr(), th.data_ptr(), c.data_ptr(), tc.data_ptr(), float(eps),
                                      gz.data_ptr(), gtz.data_ptr(), *[t.data_ptr() for t in out], workspace.data_ptr(),
                                      workspace.numel(), _stream()))
    return out


def _pointwise_args(first, *rest):
    if not first.is_cuda or not first.is_contiguous():
        raise ValueError("expected contiguous device tensors")
    for t in rest:
        if t.shape != first.shape or t.dtype != first.dtype or t.device != first.device or not t.is_contiguous():
            raise ValueError("all tensors must agree in shape, dtype, device and be contiguous")
    dt = TVMATTN_F32 if first.dtype == torch.float32 else TVMATTN_BF16 if first.dtype == torch.bfloat16 else None
    if dt is None:
        raise ValueError(f"unsupported dtype {first.dtype}")
    return first.numel(), dt


def tvmattn_gelu_jvp_fwd(u, tu, out=None):
    """Returns (a, ta): the tanh-form GELU of u and its tangent gelu'(u) * tu."""
    a, ta = out if out is not None else (torch.empty_like(u), torch.empty_like(u))
    n, dt = _pointwise_args(u, tu, a, ta)
    _check(lib().tvmattn_gelu_jvp_fwd(n, dt, u.data_ptr(), tu.data_ptr(), a.data_ptr(), ta.data_ptr(), _stream()))
    return a, ta


def tvmattn_gelu_jvp_bwd(u, tu, ga, gta, out=None):
    """Returns (gu, gtu), the gradient of <ga, a> + <gta, ta>."""
    gu, gtu = out if out is not None else (torch.empty_like(u), torch.empty_like(u))
    n, dt = _pointwise_args(u, tu, ga, gta, gu, gtu)
    _check(lib().tvmattn_gelu_jvp_bwd(n, dt, u.data_ptr(), tu.data_ptr(), ga.data_ptr(), gta.data_ptr(), gu.data_ptr(),
                                      gtu.data_ptr(), _stream()))
    return gu, gtu


def _rows(t, cols, what):
    """(R, pitch) of a tensor used as R rows of `cols` elements: a contiguous [..., cols] tensor, or a 2-D [R, cols]
    view with unit inner stride and any row pitch (a slice of a wider buffer)."""
    if not t.is_cuda or t.shape[-1] != cols or t.stride(-1) != 1:
        raise ValueError(f"{what}: expected device tensors [..., {cols}] with unit inner stride")
    if t.is_contiguous():
        return t.numel() // cols, cols
    if t.dim() == 2:
        return t.shape[0], t.stride(0)
    raise ValueError(f"{what}: a non-contiguous tensor must be given as a 2-D [R, {cols}] view")


def _linear_args(x, tx, w, bias):
    if w.dim() != 2 or w.dtype != x.dtype or not w.is_contiguous() or w.device != x.device:
        raise ValueError("the weight must be a contiguous [F, K] tensor of x's dtype on its device")
    F, K = w.shape
    R, ldx = _rows(x, K, "x")
    if tx.shape != x.shape or tx.dtype != x.dtype or tx.stride() != x.stride() or tx.device != x.device:
        raise ValueError("x and its tangent must agree in shape, dtype and layout")
    if bias is not None and (bias.shape != (F,) or bias.dtype != x.dtype or not bias.is_contiguous()
                             or bias.device != x.device):
        raise ValueError("the bias must be a contiguous [F] tensor of x's dtype on its device")
    dt = TVMATTN_F32 if x.dtype == torch.float32 else TVMATTN_BF16 if x.dtype == torch.bfloat16 else None
    if dt is None:
        raise ValueError(f"unsupported dtype {x.dtype}")
    return R, K, F, dt, ldx


def tvmattn_linear_jvp_fwd(x, tx, w, bias=None, out=None):
    """Returns (y, ty): x W^T + b and tx W^T, for x, tx [..., K] (or 2-D [R, K] views with a row pitch) and w [F, K].
    `out`: preallocated (y, ty), contiguous [..., F] or 2-D [R, F] views with a row pitch."""
    R, K, F, dt, ldx = _linear_args(x, tx, w, bias)
    if out is None:
        shape = x.shape[:-1] + (F,)
        out = (torch.empty(shape, dtype=x.dtype, device=x.device), torch.empty(shape, dtype=x.dtype, device=x.device))
    y, ty = out
    Ry, ldy = _rows(y, F, "y")
    if Ry != R or ty.shape != y.shape or ty.stride() != y.stride() or y.dtype != x.dtype or ty.dtype != x.dtype:
        raise ValueError("outputs must be two [R, F] tensors of x's dtype and one layout")
    _check(lib().tvmattn_linear_jvp_fwd(R, K, F, dt, x.data_ptr(), tx.data_ptr(), ldx, w.data_ptr(), _ptr(bias),
                                        y.data_ptr(), ty.data_ptr(), ldy, _stream()))
    return y, ty


def tvmattn_linear_jvp_bwd_workspace_bytes(x, w):
    F, K = w.shape
    dt = TVMATTN_F32 if x.dtype == torch.float32 else TVMATTN_BF16
    return int(lib().tvmattn_linear_jvp_bwd_workspace_bytes(_rows(x, K, "x")[0], K, F, dt))


def tvmattn_linear_jvp_bwd(x, tx, w, gy, gty, bias_grad=True, out=None, workspace=None):
    """Returns (gx, gtx, gw, gbias), the gradient of <gy, y> + <gty, ty> (gbias None unless bias_grad).  `out`:
    preallocated (gx, gtx, gw, gbias or None); gx, gtx must be laid out like x."""
    R, K, F, dt, ldx = _linear_args(x, tx, w, None)
    Ry, ldy = _rows(gy, F, "gy")
    if Ry != R or gty.shape != gy.shape or gty.stride() != gy.stride() or gy.dtype != x.dtype or gty.dtype != x.dtype:
        raise ValueError("upstream gradients must be two [R, F] tensors of x's dtype and one layout")
    if out is None:
        out = (_like(x), _like(x), torch.empty_like(w), torch.empty(F, dtype=x.dtype, device=x.device) if bias_grad else None)
    gx, gtx, gw, gb = out
    for t in (gx, gtx):
        if t.shape != x.shape or t.stride() != x.stride() or t.dtype != x.dtype:
            raise ValueError("gx and gtx must be laid out like x")
    if gw.shape != w.shape or not gw.is_contiguous() or gw.dtype != w.dtype:
        raise ValueError("gw must be contiguous like w")
    need = int(lib().tvmattn_linear_jvp_bwd_workspace_bytes(R, K, F, dt))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    _check(lib().tvmattn_linear_jvp_bwd(R, K, F, dt, x.data_ptr(), tx.data_ptr(), ldx, w.data_ptr(), gy.data_ptr(),
                                        gty.data_ptr(), ldy, gx.data_ptr(), gtx.data_ptr(), gw.data_ptr(), _ptr(gb),
                                        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream()))
    return out
