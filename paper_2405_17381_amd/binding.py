"""Thin ctypes binding over the C ABI of libla.so (see include/la.h).

Argument marshalling only: every step of the method runs in the HIP kernels.
PyTorch is used for device memory and streams.  If the built library is
missing this module raises; there is no CPU fallback.
"""
from __future__ import annotations

import contextlib
import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

LA_F32, LA_BF16 = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libla.so")
EXPORTS = ("la_workspace_bytes", "la_fwd", "la_bwd", "la_fwd_state", "la_decode_step", "la_gate_norm_fwd",
           "la_gate_norm_bwd", "la_fwd_swish", "la_bwd_swish", "la_fwd_wide", "la_bwd_wide", "la_lrpe_workspace_bytes",
           "la_lrpe_rotate_fwd", "la_lrpe_rotate_bwd", "la_fwd_strided", "la_bwd_strided", "la_bwd_saved", "la_strerror", "la_plan",
           "la_profile_enable", "la_profile_collect", "la_fwd_static")
# exported for tests and tuning, declared in csrc/la_debug.h, not in include/la.h
DEBUG_EXPORTS = ("la_debug_set", "la_debug_get", "la_debug_mfma_rate")
_lib = None


class LaLayout(ctypes.Structure):
    """la_layout of include/la.h: strides in elements."""
    _fields_ = [("batch_stride", ctypes.c_longlong), ("head_stride", ctypes.c_longlong),
                ("row_stride", ctypes.c_longlong)]


class LaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, la_strerror(status), status))


def load_library():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("HIP library %s is not built; run `python -c 'import __graft_entry__ as g; "
                           "g.build()'` (or paper_2405_17381_amd/build.py) first" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    fp = ctypes.POINTER(ctypes.c_float)
    lib.la_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci]
    lib.la_workspace_bytes.restype = sz
    lib.la_fwd.argtypes = [vp, vp, vp, fp, vp, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.la_fwd.restype = ci
    lib.la_bwd.argtypes = [vp, vp, vp, fp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.la_bwd.restype = ci
    lib.la_fwd_static.argtypes = [vp, vp, vp, fp, vp, ci, ci, ci, ci, ci, vp]
    lib.la_fwd_static.restype = ci
    lib.la_debug_set.argtypes = [ctypes.c_char_p, ctypes.c_long]
    lib.la_debug_set.restype = ci
    lib.la_debug_get.argtypes = [ctypes.c_char_p]
    lib.la_debug_get.restype = ctypes.c_long
    lib.la_debug_mfma_rate.argtypes = [ci, ci, vp, vp]
    lib.la_debug_mfma_rate.restype = ci
    lib.la_fwd_swish.argtypes = lib.la_fwd.argtypes
    lib.la_fwd_swish.restype = ci
    lib.la_bwd_swish.argtypes = lib.la_bwd.argtypes
    lib.la_bwd_swish.restype = ci
    lib.la_fwd_wide.argtypes = [vp, vp, vp, fp, vp, ci, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.la_fwd_wide.restype = ci
    lib.la_bwd_wide.argtypes = [vp, vp, vp, fp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.la_bwd_wide.restype = ci
    lib.la_lrpe_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.la_lrpe_workspace_bytes.restype = sz
    lib.la_lrpe_rotate_fwd.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, vp]
    lib.la_lrpe_rotate_fwd.restype = ci
    lib.la_lrpe_rotate_bwd.argtypes = [vp, vp, vp, vp, vp, ci, vp, sz, ci, ci, ci, ci, ci, vp]
    lib.la_lrpe_rotate_bwd.restype = ci
    lp = ctypes.POINTER(LaLayout)
    lib.la_fwd_strided.argtypes = [vp, vp, vp, fp, vp, lp, lp, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.la_fwd_strided.restype = ci
    lib.la_bwd_strided.argtypes = [vp, vp, vp, fp, vp, vp, vp, vp, lp, lp, lp, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.la_bwd_strided.restype = ci
    lib.la_bwd_saved.argtypes = [vp, vp, vp, fp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.la_bwd_saved.restype = ci
    lib.la_fwd_state.argtypes = [vp, vp, vp, fp, vp, vp, vp, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.la_fwd_state.restype = ci
    lib.la_decode_step.argtypes = [vp, vp, vp, fp, vp, vp, ci, ci, ci, ci, vp]
    lib.la_decode_step.restype = ci
    cf = ctypes.c_float
    lib.la_gate_norm_fwd.argtypes = [vp, vp, vp, cf, ci, ci, ci, ci, ci, vp]
    lib.la_gate_norm_fwd.restype = ci
    lib.la_gate_norm_bwd.argtypes = [vp, vp, vp, vp, vp, cf, ci, ci, ci, ci, ci, vp]
    lib.la_gate_norm_bwd.restype = ci
    lib.la_strerror.argtypes = [ci]
    lib.la_strerror.restype = ctypes.c_char_p
    ip = ctypes.POINTER(ci)
    lib.la_plan.argtypes = [ci, ci, ci, ci, ci, ip, ip, ip]
    lib.la_plan.restype = ci
    lib.la_profile_enable.argtypes = [ci]
    lib.la_profile_enable.restype = ci
    lib.la_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_double), ip]
    lib.la_profile_collect.restype = ci
    _lib = lib
    return lib


def la_strerror(status: int) -> str:
    return load_library().la_strerror(int(status)).decode()


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return LA_F32
    if t.dtype == torch.bfloat16:
        return LA_BF16
    raise TypeError("la: tensors must be float32 or bfloat16, got %s" % t.dtype)


def _check(ts: Sequence[torch.Tensor]):
    t0 = ts[0]
    if t0.dim() != 4:
        raise ValueError("la: tensors must be [B, H, n, d]")
    for t in ts:
        if not t.is_cuda:
            raise ValueError("la: tensors must live on the GPU")
        if t.shape != t0.shape or t.dtype != t0.dtype or t.device != t0.device:
            raise ValueError("la: tensors must share shape, dtype and device")
        if not t.is_contiguous():
            raise ValueError("la: tensors must be contiguous [B, H, n, d]")


def _lam(lam, H: int):
    vals = [float(x) for x in lam]
    if len(vals) != H:
        raise ValueError("la: lambda must have H entries")
    return (ctypes.c_float * H)(*vals)


def la_workspace_bytes(B: int, H: int, n: int, d: int, dt: int, is_bwd: bool) -> int:
    return int(load_library().la_workspace_bytes(B, H, n, d, dt, 1 if is_bwd else 0))


def la_plan(B: int, H: int, n: int, d: int, dt: int) -> Tuple[int, int, int]:
    """(tile length, segment length, segments per scan) the library will use."""
    a, b, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    rc = load_library().la_plan(B, H, n, d, dt, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
    if rc != 0:
        raise LaError(rc, "la_plan")
    return a.value, b.value, c.value


def _workspace(B, H, n, d, dt, is_bwd, device, workspace: Optional[torch.Tensor]):
    need = la_workspace_bytes(B, H, n, d, dt, is_bwd)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    if workspace is None:
        return None, 0, 0
    return workspace, workspace.data_ptr(), workspace.numel() * workspace.element_size()


def la_fwd(Q, K, V, lam, O=None, workspace: Optional[torch.Tensor] = None, _entry: str = "la_fwd"):
    """O = la_fwd(Q, K, V, lambda) on the current CUDA(HIP) stream."""
    _check([Q, K, V])
    B, H, n, d = Q.shape
    if O is None:
        O = torch.empty_like(Q)
    else:
        _check([Q, O])
    dt = _dt(Q)
    ws, ws_ptr, ws_bytes = _workspace(B, H, n, d, dt, False, Q.device, workspace)
    with torch.cuda.device(Q.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = getattr(load_library(), _entry)(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _lam(lam, H),
                                             O.data_ptr(), B, H, n, d, dt, ws_ptr, ws_bytes, stream)
    if rc != 0:
        raise LaError(rc, _entry)
    return O


LA_STATIC_SCRATCH_BYTES = 64 << 20


def la_fwd_static(Q, K, V, lam, O):
    """la_fwd without a workspace: the library's static scratch holds the segment states.
    O must be given (this wrapper allocates nothing either)."""
    _check([Q, K, V, O])
    B, H, n, d = Q.shape
    with torch.cuda.device(Q.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = load_library().la_fwd_static(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _lam(lam, H),
                                          O.data_ptr(), B, H, n, d, _dt(Q), stream)
    if rc != 0:
        raise LaError(rc, "la_fwd_static")
    return O


def debug_set(name: str, value: int) -> None:
    """Set a test / tuning switch of the library (csrc/la_debug.h); 0 restores the default."""
    rc = load_library().la_debug_set(name.encode(), int(value))
    if rc != 0:
        raise LaError(rc, "la_debug_set(%s)" % name)


def debug_get(name: str) -> int:
    return int(load_library().la_debug_get(name.encode()))


def debug_mfma_rate(workgroups: int, iters: int, sink: torch.Tensor) -> int:
    """Launch the register-only MFMA loop (csrc/la_debug.h) on the current stream; returns the
    number of floating-point operations the launch executes."""
    with torch.cuda.device(sink.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = load_library().la_debug_mfma_rate(int(workgroups), int(iters), sink.data_ptr(), stream)
    if rc != 0:
        raise LaError(rc, "la_debug_mfma_rate")
    return workgroups * 4 * 4 * iters * 2 * 32 * 32 * 16


@contextlib.contextmanager
def debug(**switches):
    """`with binding.debug(lseg=512): ...` sets switches for the block and clears them after."""
    for k, v in switches.items():
        debug_set(k, 0 if v is None else v)
    try:
        yield
    finally:
        for k in switches:
            debug_set(k, 0)


def la_fwd_swish(Qp, Kp, V, lam, O=None, workspace: Optional[torch.Tensor] = None):
    """O = la_fwd(swish(Qp), swish(Kp), V, lambda), the activation applied inside the kernels."""
    return la_fwd(Qp, Kp, V, lam, O=O, workspace=workspace, _entry="la_fwd_swish")


def _check_state(kv, B, H, d, device):
    if kv is None:
        return 0
    if (not kv.is_cuda) or kv.dtype != torch.float32 or tuple(kv.shape) != (B, H, d, d) \
            or not kv.is_contiguous() or kv.device != device:
        raise ValueError("la: state must be a contiguous float32 [B, H, d, d] tensor on the same GPU")
    return kv.data_ptr()


def la_fwd_state(Q, K, V, lam, kv_in=None, kv_out=None, O=None, workspace: Optional[torch.Tensor] = None):
    """O = forward pass starting from state kv_in; the state after the last token is
    written to kv_out ([B, H, d, d] float32; either may be None; may be the same tensor)."""
    _check([Q, K, V])
    B, H, n, d = Q.shape
    if O is None:
        O = torch.empty_like(Q)
    else:
        _check([Q, O])
    dt = _dt(Q)
    p_in, p_out = _check_state(kv_in, B, H, d, Q.device), _check_state(kv_out, B, H, d, Q.device)
    ws, ws_ptr, ws_bytes = _workspace(B, H, n, d, dt, False, Q.device, workspace)
    with torch.cuda.device(Q.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = load_library().la_fwd_state(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _lam(lam, H),
                                         O.data_ptr(), p_in, p_out, B, H, n, d, dt, ws_ptr, ws_bytes, stream)
    if rc != 0:
        raise LaError(rc, "la_fwd_state")
    return O


def la_decode_step(q, k, v, lam, kv, o=None):
    """One token: kv <- lambda kv + k v^T (in place), o = q^T kv.  q, k, v: [B, H, d]."""
    for t in (q, k, v):
        if t.dim() != 3 or not t.is_cuda or not t.is_contiguous() or t.shape != q.shape or t.dtype != q.dtype:
            raise ValueError("la: q, k, v must be contiguous [B, H, d] GPU tensors of one dtype")
    B, H, d = q.shape
    o = torch.empty_like(q) if o is None else o
    if o.shape != q.shape or o.dtype != q.dtype or not o.is_cuda or not o.is_contiguous():
        raise ValueError("la: o must match q")
    p_kv = _check_state(kv, B, H, d, q.device)
    if p_kv == 0:
        raise ValueError("la: kv is required")
    with torch.cuda.device(q.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = load_library().la_decode_step(q.data_ptr(), k.data_ptr(), v.data_ptr(), _lam(lam, H),
                                           p_kv, o.data_ptr(), B, H, d, _dt(q), stream)
    if rc != 0:
        raise LaError(rc, "la_decode_step")
    return o


def la_bwd(Q, K, V, lam, dO, dQ=None, dK=None, dV=None, workspace: Optional[torch.Tensor] = None,
           _entry: str = "la_bwd"):
    """(dQ, dK, dV) = la_bwd(Q, K, V, lambda, dO) on the current stream."""
    _check([Q, K, V, dO])
    B, H, n, d = Q.shape
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(Q) if dK is None else dK
    dV = torch.empty_like(Q) if dV is None else dV
    _check([Q, dQ, dK, dV])
    dt = _dt(Q)
    ws, ws_ptr, ws_bytes = _workspace(B, H, n, d, dt, True, Q.device, workspace)
    with torch.cuda.device(Q.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = getattr(load_library(), _entry)(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _lam(lam, H),
                                             dO.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(),
                                             B, H, n, d, dt, ws_ptr, ws_bytes, stream)
    if rc != 0:
        raise LaError(rc, _entry)
    return dQ, dK, dV


def la_bwd_saved(Q, K, V, lam, dO, fwd_workspace, dQ=None, dK=None, dV=None,
                 workspace: Optional[torch.Tensor] = None):
    """la_bwd reusing the segment states that la_fwd(Q, K, V, lam, workspace=fwd_workspace) left behind."""
    _check([Q, K, V, dO])
    B, H, n, d = Q.shape
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(Q) if dK is None else dK
    dV = torch.empty_like(Q) if dV is None else dV
    _check([Q, dQ, dK, dV])
    dt = _dt(Q)
    ws, ws_ptr, ws_bytes = _workspace(B, H, n, d, dt, False, Q.device, workspace)
    fptr = fwd_workspace.data_ptr() if fwd_workspace is not None else None
    with torch.cuda.device(Q.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = load_library().la_bwd_saved(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _lam(lam, H), dO.data_ptr(),
                                         dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), fptr,
                                         B, H, n, d, dt, ws_ptr, ws_bytes, stream)
    if rc != 0:
        raise LaError(rc, "la_bwd_saved")
    return dQ, dK, dV


def la_bwd_swish(Qp, Kp, V, lam, dO, dQp=None, dKp=None, dV=None, workspace: Optional[torch.Tensor] = None):
    """Gradients of la_fwd_swish with respect to the pre-activations Qp, Kp and to V."""
    return la_bwd(Qp, Kp, V, lam, dO, dQ=dQp, dK=dKp, dV=dV, workspace=workspace, _entry="la_bwd_swish")


def _layout_of(ts: Sequence[torch.Tensor]) -> LaLayout:
    """Layout shared by [B, H, n, d]-shaped views (any batch / head / row strides, unit feature stride)."""
    t0 = ts[0]
    for t in ts:
        if t.dim() != 4 or not t.is_cuda or t.shape != t0.shape or t.dtype != t0.dtype or t.device != t0.device:
            raise ValueError("la: tensors must be [B, H, n, d] views of one shape, dtype and GPU")
        if t.stride(3) != 1 or t.stride() != t0.stride():
            raise ValueError("la: views must have unit feature stride and share their strides")
    return LaLayout(t0.stride(0), t0.stride(1), t0.stride(2))


def la_fwd_strided(Q, K, V, lam, O=None, workspace: Optional[torch.Tensor] = None):
    """la_fwd on [B, H, n, d]-shaped views with arbitrary batch / head / row strides, e.g. the
    permuted view of a [B, n, H, d] projection output.  O defaults to a view laid out like Q."""
    lin = _layout_of([Q, K, V])
    B, H, n, d = Q.shape
    if O is None:
        O = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
    lout = _layout_of([O])
    dt = _dt(Q)
    ws, ws_ptr, ws_bytes = _workspace(B, H, n, d, dt, False, Q.device, workspace)
    with torch.cuda.device(Q.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = load_library().la_fwd_strided(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _lam(lam, H), O.data_ptr(),
                                           ctypes.byref(lin), ctypes.byref(lout), B, H, n, d, dt,
                                           ws_ptr, ws_bytes, stream)
    if rc != 0:
        raise LaError(rc, "la_fwd_strided")
    return O


def la_bwd_strided(Q, K, V, lam, dO, dQ=None, dK=None, dV=None, workspace: Optional[torch.Tensor] = None):
    """la_bwd on strided [B, H, n, d]-shaped views; gradients default to views laid out like Q."""
    lin = _layout_of([Q, K, V])
    ldo = _layout_of([dO])
    B, H, n, d = Q.shape
    mk = lambda: torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
    dQ = mk() if dQ is None else dQ
    dK = mk() if dK is None else dK
    dV = mk() if dV is None else dV
    lgr = _layout_of([dQ, dK, dV])
    dt = _dt(Q)
    ws, ws_ptr, ws_bytes = _workspace(B, H, n, d, dt, True, Q.device, workspace)
    with torch.cuda.device(Q.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = load_library().la_bwd_strided(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _lam(lam, H), dO.data_ptr(),
                                           dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), ctypes.byref(lin),
                                           ctypes.byref(ldo), ctypes.byref(lgr), B, H, n, d, dt,
                                           ws_ptr, ws_bytes, stream)
    if rc != 0:
        raise LaError(rc, "la_bwd_strided")
    return dQ, dK, dV


def la_fwd_wide(Qw, Kw, V, lam, O=None, workspace: Optional[torch.Tensor] = None):
    """O = attention(Qw, Kw, V, lambda) with Qw, Kw [B,H,n,dk] and V [B,H,n,dv], dk a multiple of dv."""
    _check([Qw, Kw])
    _check([V])
    B, H, n, dv = V.shape
    dk = Qw.shape[3]
    if Qw.shape[:3] != V.shape[:3] or Qw.dtype != V.dtype:
        raise ValueError("Qw / Kw and V disagree in batch, heads, length or dtype")
    O = torch.empty_like(V) if O is None else O
    _check([V, O])
    dt = _dt(V)
    ws, ws_ptr, ws_bytes = _workspace(B, H, n, dv, dt, False, V.device, workspace)
    with torch.cuda.device(V.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = load_library().la_fwd_wide(Qw.data_ptr(), Kw.data_ptr(), V.data_ptr(), _lam(lam, H), O.data_ptr(),
                                        B, H, n, dk, dv, dt, ws_ptr, ws_bytes, stream)
    if rc != 0:
        raise LaError(rc, "la_fwd_wide")
    return O


def la_bwd_wide(Qw, Kw, V, lam, dO, dQw=None, dKw=None, dV=None, workspace: Optional[torch.Tensor] = None):
    """(dQw, dKw, dV) of la_fwd_wide."""
    _check([Qw, Kw])
    _check([V, dO])
    B, H, n, dv = V.shape
    dk = Qw.shape[3]
    if Qw.shape[:3] != V.shape[:3] or Qw.dtype != V.dtype:
        raise ValueError("Qw / Kw and V disagree in batch, heads, length or dtype")
    dQw = torch.empty_like(Qw) if dQw is None else dQw
    dKw = torch.empty_like(Qw) if dKw is None else dKw
    dV = torch.empty_like(V) if dV is None else dV
    _check([Qw, dQw, dKw])
    _check([V, dV])
    dt = _dt(V)
    ws, ws_ptr, ws_bytes = _workspace(B, H, n, dv, dt, True, V.device, workspace)
    with torch.cuda.device(V.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = load_library().la_bwd_wide(Qw.data_ptr(), Kw.data_ptr(), V.data_ptr(), _lam(lam, H), dO.data_ptr(),
                                        dQw.data_ptr(), dKw.data_ptr(), dV.data_ptr(),
                                        B, H, n, dk, dv, dt, ws_ptr, ws_bytes, stream)
    if rc != 0:
        raise LaError(rc, "la_bwd_wide")
    return dQw, dKw, dV


def _check_theta(theta, H, d, device):
    if (not theta.is_cuda or theta.device != device or theta.dtype != torch.float32
            or tuple(theta.shape) != (H, d) or not theta.is_contiguous()):
        raise ValueError("la: theta must be a contiguous float32 [H, d] tensor on the tensors' device")


def la_lrpe_workspace_bytes(B: int, H: int, n: int, d: int) -> int:
    return int(load_library().la_lrpe_workspace_bytes(B, H, n, d))


def la_lrpe_rotate_fwd(X, theta, Xw=None):
    """Xw = [X cos(t theta), X sin(t theta)] ([B, H, n, 2d]); theta: float32 [H, d] on the device."""
    _check([X])
    B, H, n, d = X.shape
    _check_theta(theta, H, d, X.device)
    if Xw is None:
        Xw = torch.empty((B, H, n, 2 * d), dtype=X.dtype, device=X.device)
    _check([Xw])
    with torch.cuda.device(X.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = load_library().la_lrpe_rotate_fwd(X.data_ptr(), theta.data_ptr(), Xw.data_ptr(), B, H, n, d, _dt(X), stream)
    if rc != 0:
        raise LaError(rc, "la_lrpe_rotate_fwd")
    return Xw


def la_lrpe_rotate_bwd(X, theta, dXw, dX=None, dtheta=None, accumulate: bool = False,
                       workspace: Optional[torch.Tensor] = None):
    """(dX, dtheta) of la_lrpe_rotate_fwd; with `accumulate` the theta gradient is added to `dtheta`."""
    _check([X])
    _check([dXw])
    B, H, n, d = X.shape
    _check_theta(theta, H, d, X.device)
    dX = torch.empty_like(X) if dX is None else dX
    _check([X, dX])
    if dtheta is None:
        if accumulate:
            raise ValueError("la: accumulate needs an existing dtheta")
        dtheta = torch.empty((H, d), dtype=torch.float32, device=X.device)
    _check_theta(dtheta, H, d, X.device)
    need = la_lrpe_workspace_bytes(B, H, n, d)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=X.device)
    with torch.cuda.device(X.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = load_library().la_lrpe_rotate_bwd(X.data_ptr(), theta.data_ptr(), dXw.data_ptr(), dX.data_ptr(),
                                               dtheta.data_ptr(), 1 if accumulate else 0, workspace.data_ptr(),
                                               workspace.numel() * workspace.element_size(),
                                               B, H, n, d, _dt(X), stream)
    if rc != 0:
        raise LaError(rc, "la_lrpe_rotate_bwd")
    return dX, dtheta


def la_gate_norm_fwd(O, U, eps: float = 0.0, Y=None):
    """Y = SRMSNorm(O) * U (norm per token over all heads and features)."""
    _check([O, U])
    B, H, n, d = O.shape
    Y = torch.empty_like(O) if Y is None else Y
    _check([O, Y])
    with torch.cuda.device(O.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = load_library().la_gate_norm_fwd(O.data_ptr(), U.data_ptr(), Y.data_ptr(), float(eps),
                                             B, H, n, d, _dt(O), stream)
    if rc != 0:
        raise LaError(rc, "la_gate_norm_fwd")
    return Y


def la_gate_norm_bwd(O, U, dY, eps: float = 0.0, dO=None, dU=None):
    """(dO, dU) of Y = SRMSNorm(O) * U."""
    _check([O, U, dY])
    B, H, n, d = O.shape
    dO = torch.empty_like(O) if dO is None else dO
    dU = torch.empty_like(O) if dU is None else dU
    _check([O, dO, dU])
    with torch.cuda.device(O.device):
        stream = torch.cuda.current_stream().cuda_stream
        rc = load_library().la_gate_norm_bwd(O.data_ptr(), U.data_ptr(), dY.data_ptr(), dO.data_ptr(),
                                             dU.data_ptr(), float(eps), B, H, n, d, _dt(O), stream)
    if rc != 0:
        raise LaError(rc, "la_gate_norm_bwd")
    return dO, dU


def la_profile_enable(on: bool) -> None:
    load_library().la_profile_enable(1 if on else 0)


def la_profile_collect() -> Tuple[float, int]:
    """(total ms, launches) of the block-scan kernel since the last collect."""
    ms, cnt = ctypes.c_double(), ctypes.c_int()
    load_library().la_profile_collect(ctypes.byref(ms), ctypes.byref(cnt))
    return ms.value, cnt.value
