"""Thin ctypes binding of the C ABI in include/la.h.

Argument marshalling only: every step of the path runs in the HIP kernels of
libla_hip.so.  PyTorch supplies device memory (tensors) and streams, nothing
else.  There is no CPU fallback: if the library is missing the import fails.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libla_hip.so")

LA_F32, LA_BF16, LA_F32_FEATURES, LA_BF16_FEATURES, LA_F32_POLY2 = 0, 1, 2, 3, 4
LA_OK, LA_ERR_NULL, LA_ERR_SHAPE, LA_ERR_UNSUPPORTED = 0, -1, -2, -3
LA_ERR_WORKSPACE, LA_ERR_HIP, LA_ERR_ALIGN, LA_ERR_ALIAS, LA_ERR_SCRATCH = -4, -5, -6, -7, -8
LA_NOALLOC_SCRATCH_BYTES = 40 << 20

EXPORTS = ("la_status_string", "la_version", "la_causal_fwd_workspace", "la_causal_bwd_workspace",
           "la_global_fwd_workspace", "la_global_bwd_workspace", "la_causal_fwd", "la_causal_fwd_state",
           "la_causal_bwd", "la_causal_bwd_state", "la_causal_fwd_bnhd", "la_causal_bwd_bnhd",
           "la_causal_fwd_state_bnhd", "la_causal_bwd_state_bnhd", "la_profile_create", "la_profile_destroy",
           "la_global_fwd", "la_global_bwd", "la_global_fwd_bnhd", "la_global_bwd_bnhd",
           "la_recurrent_step", "la_recurrent_steps", "la_causal_fwd_noalloc", "la_kernel_name", "la_profile_begin",
           "la_profile_end", "la_tuning_reload")
LA_K_COUNT = 8


class LaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python paper_2006_16236_amd/build.py "
            "or __graft_entry__.build()); this package has no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    missing = [name for name in EXPORTS if not hasattr(lib, name)]
    if missing:
        raise ImportError(f"{LIB_PATH} lacks {missing}: it was built from older sources, rebuild "
                          "it (python paper_2006_16236_amd/build.py)")
    vp, i, f, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.la_status_string.restype = ctypes.c_char_p
    lib.la_status_string.argtypes = [i]
    lib.la_version.restype = i
    lib.la_tuning_reload.restype = None
    lib.la_tuning_reload.argtypes = []
    for name in ("la_causal_fwd_workspace", "la_causal_bwd_workspace", "la_global_fwd_workspace",
                 "la_global_bwd_workspace"):
        fn = getattr(lib, name)
        fn.restype = sz
        fn.argtypes = [i, i, i, i, i, i]
    lib.la_causal_fwd.restype = i
    lib.la_causal_fwd.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, f, i, vp, sz, vp]
    lib.la_causal_fwd_noalloc.restype = i
    lib.la_causal_fwd_noalloc.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, f, i, vp]
    lib.la_causal_fwd_state.restype = i
    lib.la_causal_fwd_state.argtypes = [vp] * 9 + [i, i, i, i, i, f, i, vp, sz, vp]
    lib.la_causal_bwd.restype = i
    lib.la_causal_bwd.argtypes = [vp] * 10 + [i, i, i, i, i, f, i, vp, sz, vp]
    lib.la_causal_fwd_bnhd.restype = i
    lib.la_causal_fwd_bnhd.argtypes = lib.la_causal_fwd.argtypes
    lib.la_causal_bwd_bnhd.restype = i
    lib.la_causal_bwd_bnhd.argtypes = lib.la_causal_bwd.argtypes
    lib.la_causal_bwd_state.restype = i
    lib.la_causal_bwd_state.argtypes = [vp] * 16 + [i, i, i, i, i, f, i, vp, sz, vp]
    lib.la_causal_fwd_state_bnhd.restype = i
    lib.la_causal_fwd_state_bnhd.argtypes = lib.la_causal_fwd_state.argtypes
    lib.la_causal_bwd_state_bnhd.restype = i
    lib.la_causal_bwd_state_bnhd.argtypes = lib.la_causal_bwd_state.argtypes
    lib.la_global_fwd.restype = i
    lib.la_global_fwd.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, f, i, vp, sz, vp]
    lib.la_global_bwd.restype = i
    lib.la_global_bwd.argtypes = [vp] * 10 + [i, i, i, i, i, f, i, vp, sz, vp]
    lib.la_global_fwd_bnhd.restype = i
    lib.la_global_fwd_bnhd.argtypes = lib.la_global_fwd.argtypes
    lib.la_global_bwd_bnhd.restype = i
    lib.la_global_bwd_bnhd.argtypes = lib.la_global_bwd.argtypes
    lib.la_recurrent_step.restype = i
    lib.la_recurrent_step.argtypes = [vp] * 6 + [i, i, i, i, f, i, vp]
    lib.la_recurrent_steps.restype = i
    lib.la_recurrent_steps.argtypes = [vp] * 6 + [i, i, i, i, i, f, i, vp]
    lib.la_kernel_name.restype = ctypes.c_char_p
    lib.la_kernel_name.argtypes = [i]
    lib.la_profile_create.restype = vp
    lib.la_profile_create.argtypes = []
    lib.la_profile_destroy.restype = None
    lib.la_profile_destroy.argtypes = [vp]
    lib.la_profile_begin.restype = i
    lib.la_profile_begin.argtypes = [vp, ctypes.c_uint]
    lib.la_profile_end.restype = i
    lib.la_profile_end.argtypes = [vp, ctypes.POINTER(f), ctypes.POINTER(i)]
    return lib


_lib = _load()


def status_string(status: int) -> str:
    return _lib.la_status_string(int(status)).decode()


def la_version() -> int:
    return int(_lib.la_version())


def la_tuning_reload() -> None:
    """Have the library read its LA_* tuning variables from the environment again."""
    _lib.la_tuning_reload()


def _dtype_code(t: torch.Tensor, features=False) -> int:
    """features=True: Q and K hold feature values of a map the caller applied (no elu + 1 inside,
    gradients with respect to the features).  features="poly2": Q and K hold raw 8-vectors and
    the library applies the degree-2 polynomial map vec(x x^T) (fp32 only)."""
    if features == "poly2":
        if t.dtype != torch.float32:
            raise TypeError(f"the polynomial map takes float32 tensors, not {t.dtype}")
        return LA_F32_POLY2
    if t.dtype == torch.float32:
        return LA_F32_FEATURES if features else LA_F32
    if t.dtype == torch.bfloat16:
        return LA_BF16_FEATURES if features else LA_BF16
    raise TypeError(f"unsupported dtype {t.dtype}: float32 or bfloat16")


def _ptr(t) -> int | None:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous device tensors")
    return t.data_ptr()


def _stream(stream) -> int | None:
    if stream is None:
        stream = torch.cuda.current_stream()
    h = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
    return h or None


def _ws(ws, need: int, device):
    if ws is None:
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=device)
    return ws, ws.data_ptr(), ws.numel() * ws.element_size()


def _check(status: int, where: str) -> None:
    if status != LA_OK:
        raise LaError(status, where)


def la_causal_fwd_workspace(B, H, N, D, M, dtype_code=LA_F32) -> int:
    return int(_lib.la_causal_fwd_workspace(B, H, N, D, M, dtype_code))


def la_causal_bwd_workspace(B, H, N, D, M, dtype_code=LA_F32) -> int:
    return int(_lib.la_causal_bwd_workspace(B, H, N, D, M, dtype_code))


def la_global_fwd_workspace(B, H, N, D, M, dtype_code=LA_F32) -> int:
    return int(_lib.la_global_fwd_workspace(B, H, N, D, M, dtype_code))


def la_global_bwd_workspace(B, H, N, D, M, dtype_code=LA_F32) -> int:
    return int(_lib.la_global_bwd_workspace(B, H, N, D, M, dtype_code))


# ---- argument checks -----------------------------------------------------------------------------
# The C ABI sees pointers and sizes only: a tensor that is shorter, of another element type or on
# another device than the sizes imply would make a kernel read or write past its allocation.
# Every wrapper therefore derives the sizes from Q and V and checks every other tensor against
# them before the call (ValueError / TypeError, nothing is launched).

def _like(name, t, shape, dtype, device, optional=False):
    """`t` must be a contiguous tensor of exactly this shape, element type and device.  The
    accepting path is one expression (these checks run on every call, decode steps included)."""
    if t is None:
        if optional:
            return
        raise ValueError(f"{name} is required")
    try:
        if t.shape == shape and t.dtype is dtype and t.device == device and t.is_contiguous():
            return
    except AttributeError:
        raise TypeError(f"{name} must be a torch.Tensor") from None
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)}, expected {tuple(shape)}")
    if t.dtype != dtype:
        raise ValueError(f"{name}: dtype {t.dtype}, expected {dtype}")
    if t.device != device:
        raise ValueError(f"{name}: device {t.device}, expected {device}")
    raise ValueError(f"{name} must be contiguous")


def _bytes(name, t, device):
    """A workspace: any contiguous tensor on the same device (its size is passed along)."""
    if t is None:
        return
    try:
        if t.device == device and t.is_contiguous():
            return
    except AttributeError:
        pass
    raise ValueError(f"{name} must be a contiguous tensor on {device}")


class _Sizes:
    """B, H, N, D, M and the shapes that follow from Q and V ([B,H,N,.], or [B,N,H,.] when
    token_major); `features` selects the element-type code."""

    def __init__(self, Q, V, token_major=False, features=False):
        try:
            qs, vs = Q.shape, V.shape
        except AttributeError:
            raise TypeError("Q and V must be torch.Tensors") from None
        if len(qs) != 4 or len(vs) != 4:
            raise ValueError("Q and V must have four dimensions")
        self.t = _dtype_code(Q, features)
        if token_major:
            B, N, H, D = qs
        else:
            B, H, N, D = qs
        M = vs[3]
        self.B, self.H, self.N, self.D, self.M = B, H, N, D, M
        self.qk = qs
        self.v = (qs[0], qs[1], qs[2], M)
        self.rows = (B, H, N)                             # den: always [B, H, N]
        self.dtype, self.dev = Q.dtype, Q.device
        self.dims = (B, H, N, D, M)
        self.C = D * D if self.t == LA_F32_POLY2 else D       # feature width (sizes the states)

    @property
    def S(self):
        return (self.B, self.H, self.C, self.M)

    @property
    def z(self):
        return (self.B, self.H, self.C)

    def inputs(self, Q, K, V):
        if not Q.is_contiguous():
            raise ValueError("Q must be contiguous")
        _like("K", K, self.qk, self.dtype, self.dev)
        _like("V", V, self.v, self.dtype, self.dev)

    def forward(self, Q, K, V, O, den):
        try:    # the accepting path in one expression; the named checks below find what is wrong
            qk, vv, dt, dev = self.qk, self.v, self.dtype, self.dev
            if (Q.is_contiguous() and K.shape == qk and K.dtype is dt and K.device == dev and K.is_contiguous()
                    and V.shape == vv and V.dtype is dt and V.device == dev and V.is_contiguous()
                    and O.shape == vv and O.dtype is dt and O.device == dev and O.is_contiguous()
                    and (den is None or (den.shape == self.rows and den.dtype is torch.float32
                                         and den.device == dev and den.is_contiguous()))):
                return
        except AttributeError:
            pass
        self.inputs(Q, K, V)
        _like("O", O, self.v, self.dtype, self.dev)
        _like("den", den, self.rows, torch.float32, self.dev, optional=True)

    def backward(self, Q, K, V, O, den, dO, dQ, dK, dV, fwd_ws):
        try:
            qk, vv, dt, dev = self.qk, self.v, self.dtype, self.dev
            if (O is None and fwd_ws is not None and den is not None
                    and Q.is_contiguous() and K.shape == qk and K.dtype is dt and K.device == dev and K.is_contiguous()
                    and V.shape == vv and V.dtype is dt and V.device == dev and V.is_contiguous()
                    and dO.shape == vv and dO.dtype is dt and dO.device == dev and dO.is_contiguous()
                    and dQ.shape == qk and dQ.dtype is dt and dQ.device == dev and dQ.is_contiguous()
                    and dK.shape == qk and dK.dtype is dt and dK.device == dev and dK.is_contiguous()
                    and dV.shape == vv and dV.dtype is dt and dV.device == dev and dV.is_contiguous()
                    and den.shape == self.rows and den.dtype is torch.float32 and den.device == dev
                    and den.is_contiguous() and fwd_ws.device == dev and fwd_ws.is_contiguous()):
                return
        except AttributeError:
            pass
        self.inputs(Q, K, V)
        _like("O", O, self.v, self.dtype, self.dev, optional=True)
        _like("den", den, self.rows, torch.float32, self.dev, optional=True)
        _like("dO", dO, self.v, self.dtype, self.dev)
        _like("dQ", dQ, self.qk, self.dtype, self.dev)
        _like("dK", dK, self.qk, self.dtype, self.dev)
        _like("dV", dV, self.v, self.dtype, self.dev)
        _bytes("fwd_ws", fwd_ws, self.dev)

    def state(self, **pairs):
        """fp32 state tensors by name: S-like [B,H,D,M] for names starting with S / dS, z-like
        [B,H,D] otherwise; all optional."""
        for name, t in pairs.items():
            shape = self.S if name.lstrip("d").startswith("S") else self.z
            _like(name, t, shape, torch.float32, self.dev, optional=True)


def _fwd_ws_bytes(fwd_ws, need, name):
    """A forward workspace handed to a backward must be at least as large as the forward's query."""
    if fwd_ws is not None and fwd_ws.numel() * fwd_ws.element_size() < need:
        raise ValueError(f"{name}: fwd_ws holds {fwd_ws.numel() * fwd_ws.element_size()} bytes, the forward "
                         f"of these sizes uses {need}")


def la_causal_fwd(Q, K, V, O, den=None, eps=1e-6, ws=None, stream=None, features=False):
    """O [B,H,N,M] <- causal linear attention of Q, K [B,H,N,D], V [B,H,N,M]; den [B,H,N] fp32
    (optional) receives the denominators.  Enqueues on `stream` (default: torch's current)."""
    sz = _Sizes(Q, V, features=features)
    sz.forward(Q, K, V, O, den)
    _bytes("ws", ws, sz.dev)
    ws, wp, wb = _ws(ws, la_causal_fwd_workspace(*sz.dims, sz.t), Q.device)
    _check(_lib.la_causal_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(den), *sz.dims,
                              float(eps), sz.t, wp, wb, _stream(stream)), "la_causal_fwd")
    return ws


def la_causal_fwd_noalloc(Q, K, V, O, den=None, eps=1e-6, stream=None, features=False):
    """la_causal_fwd without a workspace argument: the segment states live in the library's
    built-in scratch array (LA_NOALLOC_SCRATCH_BYTES); nothing is allocated by the call."""
    sz = _Sizes(Q, V, features=features)
    sz.forward(Q, K, V, O, den)
    _check(_lib.la_causal_fwd_noalloc(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(den), *sz.dims,
                                      float(eps), sz.t, _stream(stream)), "la_causal_fwd_noalloc")


def la_causal_fwd_state(Q, K, V, O, den=None, S0=None, z0=None, S1=None, z1=None, eps=1e-6, ws=None,
                        stream=None, features=False, token_major=False):
    """Causal forward that starts from the state (S0, z0) (None: zero) and returns the state
    after the last token in (S1, z1) (None: not wanted); all four fp32 [B,H,D,M] / [B,H,D].
    token_major: Q, K, V, O are [B,N,H,.] (la_causal_fwd_state_bnhd)."""
    sz = _Sizes(Q, V, token_major=token_major, features=features)
    sz.forward(Q, K, V, O, den)
    sz.state(S0=S0, z0=z0, S1=S1, z1=z1)
    _bytes("ws", ws, sz.dev)
    ws, wp, wb = _ws(ws, la_causal_fwd_workspace(*sz.dims, sz.t), Q.device)
    fn = _lib.la_causal_fwd_state_bnhd if token_major else _lib.la_causal_fwd_state
    _check(fn(_ptr(Q), _ptr(K), _ptr(V), _ptr(S0), _ptr(z0), _ptr(O), _ptr(den), _ptr(S1), _ptr(z1),
              *sz.dims, float(eps), sz.t, wp, wb, _stream(stream)), "la_causal_fwd_state")
    return ws


def la_causal_bwd(Q, K, V, O, den, dO, dQ, dK, dV, eps=1e-6, ws=None, stream=None, fwd_ws=None,
                  features=False):
    """dQ, dK, dV <- gradients of causal linear attention for upstream dO; O and den are the
    forward results (den None: recomputed; O is not read and may be None).  fwd_ws (optional) is
    the workspace tensor la_causal_fwd returned for the same call: its segment states are reused."""
    sz = _Sizes(Q, V, features=features)
    sz.backward(Q, K, V, O, den, dO, dQ, dK, dV, fwd_ws)
    _fwd_ws_bytes(fwd_ws, la_causal_fwd_workspace(*sz.dims, sz.t), "la_causal_bwd")
    _bytes("ws", ws, sz.dev)
    ws, wp, wb = _ws(ws, la_causal_bwd_workspace(*sz.dims, sz.t), Q.device)
    _check(_lib.la_causal_bwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(den), _ptr(fwd_ws),
                              _ptr(dO), _ptr(dQ), _ptr(dK), _ptr(dV), *sz.dims, float(eps), sz.t,
                              wp, wb, _stream(stream)), "la_causal_bwd")
    return ws


def la_causal_fwd_bnhd(Q, K, V, O, den=None, eps=1e-6, ws=None, stream=None, features=False):
    """la_causal_fwd on token-major tensors: Q, K [B,N,H,D], V, O [B,N,H,M]; den stays [B,H,N]."""
    sz = _Sizes(Q, V, token_major=True, features=features)
    sz.forward(Q, K, V, O, den)
    _bytes("ws", ws, sz.dev)
    ws, wp, wb = _ws(ws, la_causal_fwd_workspace(*sz.dims, sz.t), Q.device)
    _check(_lib.la_causal_fwd_bnhd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(den), *sz.dims,
                                   float(eps), sz.t, wp, wb, _stream(stream)), "la_causal_fwd_bnhd")
    return ws


def la_causal_bwd_bnhd(Q, K, V, O, den, dO, dQ, dK, dV, eps=1e-6, ws=None, stream=None, fwd_ws=None,
                       features=False):
    """la_causal_bwd on token-major tensors ([B,N,H,.]; den [B,H,N]); fwd_ws from
    la_causal_fwd_bnhd."""
    sz = _Sizes(Q, V, token_major=True, features=features)
    sz.backward(Q, K, V, O, den, dO, dQ, dK, dV, fwd_ws)
    _fwd_ws_bytes(fwd_ws, la_causal_fwd_workspace(*sz.dims, sz.t), "la_causal_bwd_bnhd")
    _bytes("ws", ws, sz.dev)
    ws, wp, wb = _ws(ws, la_causal_bwd_workspace(*sz.dims, sz.t), Q.device)
    _check(_lib.la_causal_bwd_bnhd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(den), _ptr(fwd_ws),
                                   _ptr(dO), _ptr(dQ), _ptr(dK), _ptr(dV), *sz.dims,
                                   float(eps), sz.t, wp, wb, _stream(stream)), "la_causal_bwd_bnhd")
    return ws


def la_causal_bwd_state(Q, K, V, O, den, dO, dQ, dK, dV, S0=None, z0=None, dS1=None, dz1=None,
                        dS0=None, dz0=None, eps=1e-6, ws=None, stream=None, fwd_ws=None,
                        features=False, token_major=False):
    """la_causal_bwd for a piece whose forward started from (S0, z0): (dS1, dz1) is the gradient
    arriving at the state after the last token (None: zero), (dS0, dz0) receives the gradient
    for (S0, z0) (None: not wanted); all fp32 [B,H,D,M] / [B,H,D].  token_major: the N-sized
    tensors are [B,N,H,.] (la_causal_bwd_state_bnhd)."""
    sz = _Sizes(Q, V, token_major=token_major, features=features)
    sz.backward(Q, K, V, O, den, dO, dQ, dK, dV, fwd_ws)
    sz.state(S0=S0, z0=z0, dS1=dS1, dz1=dz1, dS0=dS0, dz0=dz0)
    _fwd_ws_bytes(fwd_ws, la_causal_fwd_workspace(*sz.dims, sz.t), "la_causal_bwd_state")
    _bytes("ws", ws, sz.dev)
    ws, wp, wb = _ws(ws, la_causal_bwd_workspace(*sz.dims, sz.t), Q.device)
    fn = _lib.la_causal_bwd_state_bnhd if token_major else _lib.la_causal_bwd_state
    _check(fn(_ptr(Q), _ptr(K), _ptr(V), _ptr(S0), _ptr(z0), _ptr(O), _ptr(den), _ptr(fwd_ws),
              _ptr(dO), _ptr(dS1), _ptr(dz1), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dS0), _ptr(dz0),
              *sz.dims, float(eps), sz.t, wp, wb, _stream(stream)), "la_causal_bwd_state")
    return ws


def la_global_fwd(Q, K, V, O, eps=1e-6, ws=None, stream=None, den=None, features=False):
    """O <- non-causal linear attention (every query sees every key); den [B,H,N] fp32
    (optional) receives the denominators."""
    sz = _Sizes(Q, V, features=features)
    sz.forward(Q, K, V, O, den)
    _bytes("ws", ws, sz.dev)
    ws, wp, wb = _ws(ws, la_global_fwd_workspace(*sz.dims, sz.t), Q.device)
    _check(_lib.la_global_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(den), *sz.dims,
                              float(eps), sz.t, wp, wb, _stream(stream)), "la_global_fwd")
    return ws


def la_global_bwd(Q, K, V, O, den, dO, dQ, dK, dV, eps=1e-6, ws=None, stream=None, fwd_ws=None,
                  features=False):
    """dQ, dK, dV <- gradients of non-causal linear attention for upstream dO; O and den are the
    results of la_global_fwd (den None: recomputed; O is not read and may be None).  fwd_ws
    (optional) is the workspace tensor la_global_fwd returned for the same call."""
    sz = _Sizes(Q, V, features=features)
    sz.backward(Q, K, V, O, den, dO, dQ, dK, dV, fwd_ws)
    _fwd_ws_bytes(fwd_ws, la_global_fwd_workspace(*sz.dims, sz.t), "la_global_bwd")
    _bytes("ws", ws, sz.dev)
    ws, wp, wb = _ws(ws, la_global_bwd_workspace(*sz.dims, sz.t), Q.device)
    _check(_lib.la_global_bwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(den), _ptr(fwd_ws),
                              _ptr(dO), _ptr(dQ), _ptr(dK), _ptr(dV), *sz.dims, float(eps), sz.t,
                              wp, wb, _stream(stream)), "la_global_bwd")
    return ws


def la_global_fwd_bnhd(Q, K, V, O, eps=1e-6, ws=None, stream=None, den=None, features=False):
    """la_global_fwd on token-major tensors: Q, K [B,N,H,D], V, O [B,N,H,M]; den stays [B,H,N]."""
    sz = _Sizes(Q, V, token_major=True, features=features)
    sz.forward(Q, K, V, O, den)
    _bytes("ws", ws, sz.dev)
    ws, wp, wb = _ws(ws, la_global_fwd_workspace(*sz.dims, sz.t), Q.device)
    _check(_lib.la_global_fwd_bnhd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(den), *sz.dims,
                                   float(eps), sz.t, wp, wb, _stream(stream)), "la_global_fwd_bnhd")
    return ws


def la_global_bwd_bnhd(Q, K, V, O, den, dO, dQ, dK, dV, eps=1e-6, ws=None, stream=None, fwd_ws=None,
                       features=False):
    """la_global_bwd on token-major tensors ([B,N,H,.]; den [B,H,N]); fwd_ws from
    la_global_fwd_bnhd."""
    sz = _Sizes(Q, V, token_major=True, features=features)
    sz.backward(Q, K, V, O, den, dO, dQ, dK, dV, fwd_ws)
    _fwd_ws_bytes(fwd_ws, la_global_fwd_workspace(*sz.dims, sz.t), "la_global_bwd_bnhd")
    _bytes("ws", ws, sz.dev)
    ws, wp, wb = _ws(ws, la_global_bwd_workspace(*sz.dims, sz.t), Q.device)
    _check(_lib.la_global_bwd_bnhd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(den), _ptr(fwd_ws),
                                   _ptr(dO), _ptr(dQ), _ptr(dK), _ptr(dV), *sz.dims,
                                   float(eps), sz.t, wp, wb, _stream(stream)), "la_global_bwd_bnhd")
    return ws


def _step_checks(q, k, v, S, z, out, lead, features):
    """Shapes of the decode calls: q, k [*lead, B, H, D], v, out [*lead, B, H, M]."""
    try:
        qs, vs = q.shape, v.shape
    except AttributeError:
        raise TypeError("q and v must be torch.Tensors") from None
    if len(qs) != 3 + lead or len(vs) != 3 + lead:
        raise ValueError(f"q and v must have {3 + lead} dimensions")
    t = _dtype_code(q, features)
    B, H, D = qs[lead:]
    M = vs[-1]
    C = D * D if t == LA_F32_POLY2 else D          # feature width (sizes the state)
    dev, dt = q.device, q.dtype
    vshape = tuple(qs[:-1]) + (M,)
    try:        # the accepting path: one expression, no calls (this runs before every decode step)
        if (q.is_contiguous() and k.shape == qs and k.dtype is dt and k.device == dev and k.is_contiguous()
                and v.shape == vshape and v.dtype is dt and v.device == dev and v.is_contiguous()
                and out.shape == vshape and out.dtype is dt and out.device == dev and out.is_contiguous()
                and S.shape == (B, H, C, M) and S.dtype is torch.float32 and S.device == dev and S.is_contiguous()
                and z.shape == (B, H, C) and z.dtype is torch.float32 and z.device == dev and z.is_contiguous()):
            return t, B, H, D, M
    except AttributeError:
        pass
    if not q.is_contiguous():
        raise ValueError("q must be contiguous")
    _like("k", k, qs, dt, dev)
    _like("v", v, vshape, dt, dev)
    _like("out", out, vshape, dt, dev)
    _like("S", S, (B, H, C, M), torch.float32, dev)
    _like("z", z, (B, H, C), torch.float32, dev)
    return t, B, H, D, M


def la_recurrent_step(q, k, v, S, z, out, eps=1e-6, stream=None, features=False):
    """One decode step for q, k [B,H,D], v [B,H,M]: S [B,H,D,M], z [B,H,D] (fp32) are updated
    in place, out [B,H,M] receives the attention output of the new token."""
    t, B, H, D, M = _step_checks(q, k, v, S, z, out, 0, features)
    _check(_lib.la_recurrent_step(_ptr(q), _ptr(k), _ptr(v), _ptr(S), _ptr(z), _ptr(out), B, H, D,
                                  M, float(eps), t, _stream(stream)),
           "la_recurrent_step")


def la_recurrent_steps(q, k, v, S, z, out, eps=1e-6, stream=None, features=False):
    """T decode steps in one launch: q, k [T,B,H,D], v, out [T,B,H,M]; S, z updated in place."""
    t, B, H, D, M = _step_checks(q, k, v, S, z, out, 1, features)
    T = q.shape[0]
    _check(_lib.la_recurrent_steps(_ptr(q), _ptr(k), _ptr(v), _ptr(S), _ptr(z), _ptr(out), T, B, H,
                                   D, M, float(eps), t, _stream(stream)),
           "la_recurrent_steps")


def la_kernel_name(kernel_id: int) -> str:
    return _lib.la_kernel_name(int(kernel_id)).decode()


class Profile:
    """Owner of one la_profile object of the library (HIP events around selected launches made by
    the thread that calls begin())."""

    def __init__(self):
        self._h = _lib.la_profile_create()
        if not self._h:
            raise MemoryError("la_profile_create failed")

    def begin(self, mask: int = (1 << LA_K_COUNT) - 1) -> None:
        _check(_lib.la_profile_begin(self._h, int(mask)), "la_profile_begin")

    def end(self) -> dict:
        """Wait for the recorded events; {kernel name: (total ms, launches)} for kernels that ran."""
        ms = (ctypes.c_float * LA_K_COUNT)()
        n = (ctypes.c_int * LA_K_COUNT)()
        _check(_lib.la_profile_end(self._h, ms, n), "la_profile_end")
        return {la_kernel_name(k): (float(ms[k]), int(n[k])) for k in range(LA_K_COUNT) if n[k] > 0}

    def close(self) -> None:
        if self._h:
            _lib.la_profile_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


_default_profile = None


def la_profile_begin(mask: int = (1 << LA_K_COUNT) - 1) -> None:
    """Bracket every launch (made by this thread) of the kernels selected by `mask` with HIP
    events, using one Profile object kept by this module."""
    global _default_profile
    if _default_profile is None:
        _default_profile = Profile()
    _default_profile.begin(mask)


def la_profile_end() -> dict:
    """{kernel name: (total ms, launches)} since la_profile_begin."""
    if _default_profile is None:
        raise RuntimeError("la_profile_end without la_profile_begin")
    return _default_profile.end()


def raw():
    """The ctypes library handle, for tests of the raw C ABI (error paths)."""
    return _lib
