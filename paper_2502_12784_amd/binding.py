"""Thin ctypes binding of the C ABI in ``include/spark_mha.h``.

Argument marshalling only: every step of the attention path runs in the HIP
kernels of ``libspark_mha.so``.  torch is used for device memory and for the
current stream.  There is no fallback: if the library is missing or a call
fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libspark_mha.so")

SPARK_F16 = 0
SPARK_BF16 = 1

EXPORTS = ("spark_mha_fwd", "spark_mha_bwd", "spark_mha_bwd_marked",
           "spark_mha_bwd_workspace_bytes", "spark_mha_cross_fwd", "spark_mha_cross_bwd",
           "spark_mha_cross_bwd_workspace_bytes", "spark_mha_dropout_fwd", "spark_mha_dropout_bwd",
           "spark_dropout_threshold", "spark_dropout_mask", "spark_mha_strided_fwd",
           "spark_mha_strided_bwd", "spark_status_str", "spark_mha_bwd_static",
           "spark_mha_bwd_static_max_rows", "spark_layout_probe", "spark_mha_bwd_atomic",
           "spark_mha_bwd_atomic_workspace_bytes", "spark_mha_dropout_bwd_marked")

_lib = None


class Strides(ctypes.Structure):
    """spark_strides_t: element strides of the batch, head and row indices."""
    _fields_ = [("batch", ctypes.c_longlong), ("head", ctypes.c_longlong), ("row", ctypes.c_longlong)]


class SparkError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("spark_mha: %s (status %d)" % (message, status))
        self.status = status


def library_is_stale() -> bool:
    """True if the shared library is missing or older than any of the sources it is built from."""
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    csrc = os.path.join(HERE, "csrc")
    sources = [os.path.join(csrc, f) for f in os.listdir(csrc) if f.endswith((".hip", ".hpp", ".h"))]
    sources.append(os.path.join(os.path.dirname(HERE), "include", "spark_mha.h"))
    return any(os.path.getmtime(f) > built for f in sources if os.path.exists(f))


def load_library() -> ctypes.CDLL:
    """Load the in-tree shared library; build it first if it is missing or older than its sources
    (an edit under csrc/ must never be tested or timed against the previous binary)."""
    global _lib
    if _lib is not None:
        return _lib
    if library_is_stale():
        from .build import build_library
        build_library()
    # torch first: its wheel brings its own copy of the HIP runtime, and the streams and pointers this
    # binding passes belong to that copy.  Loaded after torch, the library binds to the runtime that
    # is already in the process; loaded before it, it would pull in a second one and every launch
    # on a torch stream would be refused.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i, f = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lib.spark_mha_fwd.restype = i
    lib.spark_mha_fwd.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, f, i, i, vp]
    lib.spark_mha_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.spark_mha_bwd_workspace_bytes.argtypes = [i, i, i, i, i]
    lib.spark_mha_bwd.restype = i
    lib.spark_mha_bwd.argtypes = [vp] * 10 + [ctypes.c_size_t, i, i, i, i, f, i, i, vp]
    lib.spark_mha_cross_fwd.restype = i
    lib.spark_mha_cross_fwd.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, f, i, i, vp]
    lib.spark_mha_cross_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.spark_mha_cross_bwd_workspace_bytes.argtypes = [i, i, i, i, i, i]
    lib.spark_mha_cross_bwd.restype = i
    lib.spark_mha_cross_bwd.argtypes = [vp] * 10 + [ctypes.c_size_t, i, i, i, i, i, f, i, i, vp]
    u64, u32 = ctypes.c_uint64, ctypes.c_uint32
    lib.spark_mha_dropout_fwd.restype = i
    lib.spark_mha_dropout_fwd.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, f, i, f, u64, u32, i, vp]
    lib.spark_mha_dropout_bwd.restype = i
    lib.spark_mha_dropout_bwd.argtypes = ([vp] * 10 + [ctypes.c_size_t, i, i, i, i, i, f, i, f, u64,
                                                      u32, i, vp])
    lib.spark_mha_dropout_bwd_marked.restype = i
    lib.spark_mha_dropout_bwd_marked.argtypes = lib.spark_mha_dropout_bwd.argtypes + [ctypes.POINTER(vp)]
    lib.spark_dropout_threshold.restype = i
    lib.spark_dropout_threshold.argtypes = [f]
    lib.spark_dropout_mask.restype = i
    lib.spark_dropout_mask.argtypes = [vp, i, i, i, i, f, u64, u32, vp]
    sp = ctypes.POINTER(Strides)
    lib.spark_mha_strided_fwd.restype = i
    lib.spark_mha_strided_fwd.argtypes = [vp] * 5 + [sp] * 4 + [i, i, i, i, i, f, i, f, u64, u32, i, vp]
    lib.spark_mha_strided_bwd.restype = i
    lib.spark_mha_strided_bwd.argtypes = ([vp] * 9 + [sp] * 8 + [vp, ctypes.c_size_t, i, i, i, i, i, f, i,
                                                             f, u64, u32, i, vp])
    lib.spark_mha_bwd_marked.restype = i
    lib.spark_mha_bwd_marked.argtypes = lib.spark_mha_bwd.argtypes + [ctypes.POINTER(vp)]
    lib.spark_mha_bwd_static.restype = i
    lib.spark_mha_bwd_static.argtypes = [vp] * 9 + [i, i, i, i, f, i, i, vp]
    lib.spark_mha_bwd_static_max_rows.restype = ctypes.c_size_t
    lib.spark_mha_bwd_static_max_rows.argtypes = []
    lib.spark_mha_bwd_atomic_workspace_bytes.restype = ctypes.c_size_t
    lib.spark_mha_bwd_atomic_workspace_bytes.argtypes = [i, i, i, i, i, i]
    lib.spark_mha_bwd_atomic.restype = i
    lib.spark_mha_bwd_atomic.argtypes = lib.spark_mha_cross_bwd.argtypes
    lib.spark_layout_probe.restype = i
    lib.spark_layout_probe.argtypes = [vp, i, vp]
    lib.spark_status_str.restype = ctypes.c_char_p
    lib.spark_status_str.argtypes = [i]
    _lib = lib
    return lib


def status_str(status: int) -> str:
    return load_library().spark_status_str(int(status)).decode()


def _check(status: int) -> None:
    if status != 0:
        raise SparkError(status, status_str(status))


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float16:
        return SPARK_F16
    if t.dtype == torch.bfloat16:
        return SPARK_BF16
    raise SparkError(-3, "tensors must be float16 or bfloat16")


def _require(t, shape, dtype, name):
    if not t.is_cuda:
        raise ValueError("%s must be a device tensor" % name)
    if tuple(t.shape) != tuple(shape) or t.dtype != dtype or not t.is_contiguous():
        raise ValueError("%s must be a contiguous %s tensor of shape %s" % (name, dtype, tuple(shape)))


def _stream_ptr():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def spark_mha_fwd(Q, K, V, scale: float, causal: bool, O=None, LSE=None):
    """O, LSE = fused attention forward of [B,H,N,d] device tensors on the current stream."""
    import torch
    lib = load_library()
    B, H, N, d = Q.shape
    for t, n in ((Q, "Q"), (K, "K"), (V, "V")):
        _require(t, (B, H, N, d), Q.dtype, n)
    if O is None:
        O = torch.empty_like(Q)
    if LSE is None:
        LSE = torch.empty((B, H, N), dtype=torch.float32, device=Q.device)
    _require(O, (B, H, N, d), Q.dtype, "O")
    _require(LSE, (B, H, N), torch.float32, "LSE")
    _check(lib.spark_mha_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), LSE.data_ptr(),
                             B, H, N, d, float(scale), int(bool(causal)), _dtype_code(Q), _stream_ptr()))
    return O, LSE


def spark_mha_bwd_workspace_bytes(B: int, H: int, N: int, d: int, dtype_code: int) -> int:
    return int(load_library().spark_mha_bwd_workspace_bytes(B, H, N, d, dtype_code))


def spark_mha_cross_bwd_workspace_bytes(B: int, H: int, Nq: int, Nk: int, d: int,
                                        dtype_code: int) -> int:
    return int(load_library().spark_mha_cross_bwd_workspace_bytes(B, H, Nq, Nk, d, dtype_code))


def spark_dropout_threshold(p_drop: float) -> int:
    return int(load_library().spark_dropout_threshold(float(p_drop)))


def spark_dropout_mask(B: int, H: int, Nq: int, Nk: int, p_drop: float, seed: int, offset: int,
                       device="cuda"):
    """The keep mask [B,H,Nq,Nk] (uint8, 1 = keep) that the dropout kernels regenerate."""
    import torch
    M = torch.empty((B, H, Nq, Nk), dtype=torch.uint8, device=device)
    _check(load_library().spark_dropout_mask(M.data_ptr(), B, H, Nq, Nk, float(p_drop), int(seed),
                                             int(offset), _stream_ptr()))
    return M


def spark_mha_cross_fwd(Q, K, V, scale: float, causal: bool = False, O=None, LSE=None, dropout=None):
    """O, LSE for Q [B,H,Nq,d] attending to K, V [B,H,Nk,d] (Nq and Nk may differ).
    dropout: None, or (p_drop, seed, offset) -> spark_mha_dropout_fwd."""
    import torch
    lib = load_library()
    B, H, Nq, d = Q.shape
    Nk = K.shape[2]
    _require(Q, (B, H, Nq, d), Q.dtype, "Q")
    for t, n in ((K, "K"), (V, "V")):
        _require(t, (B, H, Nk, d), Q.dtype, n)
    if O is None:
        O = torch.empty_like(Q)
    if LSE is None:
        LSE = torch.empty((B, H, Nq), dtype=torch.float32, device=Q.device)
    _require(O, (B, H, Nq, d), Q.dtype, "O")
    _require(LSE, (B, H, Nq), torch.float32, "LSE")
    if dropout is None:
        _check(lib.spark_mha_cross_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                       LSE.data_ptr(), B, H, Nq, Nk, d, float(scale),
                                       int(bool(causal)), _dtype_code(Q), _stream_ptr()))
    else:
        p_drop, seed, offset = dropout
        _check(lib.spark_mha_dropout_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                         LSE.data_ptr(), B, H, Nq, Nk, d, float(scale),
                                         int(bool(causal)), float(p_drop), int(seed), int(offset),
                                         _dtype_code(Q), _stream_ptr()))
    return O, LSE


def spark_mha_dropout_fwd(Q, K, V, scale: float, causal: bool, p_drop: float, seed: int,
                          offset: int, O=None, LSE=None):
    """Forward with attention dropout; the mask is a function of (p_drop, seed, offset)."""
    return spark_mha_cross_fwd(Q, K, V, scale, causal, O, LSE, dropout=(p_drop, seed, offset))


def spark_mha_dropout_bwd(Q, K, V, O, LSE, dO, scale: float, causal: bool, p_drop: float,
                          seed: int, offset: int, dQ=None, dK=None, dV=None, workspace=None, events=None):
    """Backward of spark_mha_dropout_fwd; pass the same (p_drop, seed, offset).
    ``events``: optional ``(HipEvents, first_index)`` -> spark_mha_dropout_bwd_marked."""
    return spark_mha_cross_bwd(Q, K, V, O, LSE, dO, scale, causal, dQ, dK, dV, workspace,
                               dropout=(p_drop, seed, offset), events=events)


def spark_mha_cross_bwd(Q, K, V, O, LSE, dO, scale: float, causal: bool = False, dQ=None,
                        dK=None, dV=None, workspace=None, dropout=None, events=None):
    """dQ [B,H,Nq,d], dK, dV [B,H,Nk,d] for the problem of spark_mha_cross_fwd.
    dropout: None, or (p_drop, seed, offset) -> spark_mha_dropout_bwd."""
    import torch
    lib = load_library()
    B, H, Nq, d = Q.shape
    Nk = K.shape[2]
    for t, n in ((Q, "Q"), (O, "O"), (dO, "dO")):
        _require(t, (B, H, Nq, d), Q.dtype, n)
    for t, n in ((K, "K"), (V, "V")):
        _require(t, (B, H, Nk, d), Q.dtype, n)
    _require(LSE, (B, H, Nq), torch.float32, "LSE")
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(K) if dV is None else dV
    _require(dQ, (B, H, Nq, d), Q.dtype, "dQ")
    for t, n in ((dK, "dK"), (dV, "dV")):
        _require(t, (B, H, Nk, d), Q.dtype, n)
    code = _dtype_code(Q)
    need = spark_mha_cross_bwd_workspace_bytes(B, H, Nq, Nk, d, code)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=Q.device)
    wbytes = workspace.numel() * workspace.element_size()
    ptrs = [Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), LSE.data_ptr(), dO.data_ptr(),
            dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), workspace.data_ptr(), wbytes]
    if dropout is None:
        _check(lib.spark_mha_cross_bwd(*ptrs, B, H, Nq, Nk, d, float(scale), int(bool(causal)), code,
                                       _stream_ptr()))
    else:
        p_drop, seed, offset = dropout
        tail = (B, H, Nq, Nk, d, float(scale), int(bool(causal)), float(p_drop), int(seed), int(offset),
                code, _stream_ptr())
        if events is None:
            _check(lib.spark_mha_dropout_bwd(*ptrs, *tail))
        else:
            _check(lib.spark_mha_dropout_bwd_marked(*ptrs, *tail, events[0].slice_ptr(events[1])))
    return dQ, dK, dV


def _strided(t, shape, dtype, name):
    """Check a [B,H,N,d] view whose last dimension is contiguous; return its spark_strides_t."""
    if not t.is_cuda:
        raise ValueError("%s must be a device tensor" % name)
    if tuple(t.shape) != tuple(shape) or t.dtype != dtype or t.stride(3) != 1:
        raise ValueError("%s must be a %s view of shape %s with contiguous last dimension"
                         % (name, dtype, tuple(shape)))
    return Strides(t.stride(0), t.stride(1), t.stride(2))


def spark_mha_strided_fwd(Q, K, V, scale: float, causal: bool = False, p_drop: float = 0.0,
                          seed: int = 0, offset: int = 0, O=None, LSE=None):
    """Forward on [B,H,N,d] views with arbitrary batch/head/row strides (e.g. a permuted
    [B,N,H,d] projection output, or slices of a packed QKV buffer)."""
    import torch
    lib = load_library()
    B, H, Nq, d = Q.shape
    Nk = K.shape[2]
    if O is None:
        O = torch.empty_like(Q)  # keeps Q's (dense) layout
    if LSE is None:
        LSE = torch.empty((B, H, Nq), dtype=torch.float32, device=Q.device)
    sq, so = _strided(Q, (B, H, Nq, d), Q.dtype, "Q"), _strided(O, (B, H, Nq, d), Q.dtype, "O")
    sk, sv = _strided(K, (B, H, Nk, d), Q.dtype, "K"), _strided(V, (B, H, Nk, d), Q.dtype, "V")
    _require(LSE, (B, H, Nq), torch.float32, "LSE")
    _check(lib.spark_mha_strided_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                     LSE.data_ptr(), sq, sk, sv, so, B, H, Nq, Nk, d, float(scale),
                                     int(bool(causal)), float(p_drop), int(seed), int(offset),
                                     _dtype_code(Q), _stream_ptr()))
    return O, LSE


def spark_mha_strided_bwd(Q, K, V, O, LSE, dO, scale: float, causal: bool = False,
                          p_drop: float = 0.0, seed: int = 0, offset: int = 0, dQ=None, dK=None,
                          dV=None, workspace=None):
    """Backward on strided [B,H,N,d] views; gradients default to the layouts of Q, K, V."""
    import torch
    lib = load_library()
    B, H, Nq, d = Q.shape
    Nk = K.shape[2]
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    qs, ks = (B, H, Nq, d), (B, H, Nk, d)
    st = [_strided(Q, qs, Q.dtype, "Q"), _strided(K, ks, Q.dtype, "K"), _strided(V, ks, Q.dtype, "V"),
          _strided(O, qs, Q.dtype, "O"), _strided(dO, qs, Q.dtype, "dO"), _strided(dQ, qs, Q.dtype, "dQ"),
          _strided(dK, ks, Q.dtype, "dK"), _strided(dV, ks, Q.dtype, "dV")]
    _require(LSE, (B, H, Nq), torch.float32, "LSE")
    code = _dtype_code(Q)
    need = spark_mha_cross_bwd_workspace_bytes(B, H, Nq, Nk, d, code)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=Q.device)
    wbytes = workspace.numel() * workspace.element_size()
    _check(lib.spark_mha_strided_bwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                     LSE.data_ptr(), dO.data_ptr(), dQ.data_ptr(), dK.data_ptr(),
                                     dV.data_ptr(), *st, workspace.data_ptr(), wbytes, B, H, Nq, Nk, d,
                                     float(scale), int(bool(causal)), float(p_drop), int(seed),
                                     int(offset), code, _stream_ptr()))
    return dQ, dK, dV


class HipEvents:
    """A fixed set of HIP events created through the HIP runtime itself (for
    spark_mha_bwd_marked and for timing on the stream the kernels run on)."""

    def __init__(self, n: int):
        self._hip = ctypes.CDLL("libamdhip64.so")
        self._hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self._hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self._hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self._hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p,
                                                  ctypes.c_void_p]
        self._hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.handles = (ctypes.c_void_p * n)()
        for k in range(n):
            ev = ctypes.c_void_p()
            if self._hip.hipEventCreate(ctypes.byref(ev)) != 0:
                raise RuntimeError("hipEventCreate failed")
            self.handles[k] = ev

    def record(self, k: int) -> None:
        if self._hip.hipEventRecord(self.handles[k], _stream_ptr()) != 0:
            raise RuntimeError("hipEventRecord failed")

    def synchronize(self, k: int) -> None:
        if self._hip.hipEventSynchronize(self.handles[k]) != 0:
            raise RuntimeError("hipEventSynchronize failed")

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = ctypes.c_float()
        if self._hip.hipEventElapsedTime(ctypes.byref(ms), self.handles[a], self.handles[b]) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return float(ms.value)

    def slice_ptr(self, first: int):
        """Pointer to handles[first:], as the `events` argument of spark_mha_bwd_marked."""
        return ctypes.cast(ctypes.byref(self.handles, first * ctypes.sizeof(ctypes.c_void_p)),
                           ctypes.POINTER(ctypes.c_void_p))

    def close(self) -> None:
        for h in self.handles:
            if h:
                self._hip.hipEventDestroy(h)
        self.handles = (ctypes.c_void_p * 0)()


def spark_mha_bwd(Q, K, V, O, LSE, dO, scale: float, causal: bool, dQ=None, dK=None, dV=None,
                  workspace=None, events=None):
    """dQ, dK, dV = fused attention backward on the current stream.

    ``events``: optional ``(HipEvents, first_index)``; then spark_mha_bwd_marked is called and
    records 3 events starting at that index around the two kernels (dQ, then dK/dV)."""
    import torch
    lib = load_library()
    B, H, N, d = Q.shape
    for t, n in ((Q, "Q"), (K, "K"), (V, "V"), (O, "O"), (dO, "dO")):
        _require(t, (B, H, N, d), Q.dtype, n)
    _require(LSE, (B, H, N), torch.float32, "LSE")
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(Q) if dK is None else dK
    dV = torch.empty_like(Q) if dV is None else dV
    for t, n in ((dQ, "dQ"), (dK, "dK"), (dV, "dV")):
        _require(t, (B, H, N, d), Q.dtype, n)
    code = _dtype_code(Q)
    need = spark_mha_bwd_workspace_bytes(B, H, N, d, code)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=Q.device)
    wbytes = workspace.numel() * workspace.element_size()
    args = [Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), LSE.data_ptr(),
            dO.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(),
            workspace.data_ptr(), wbytes, B, H, N, d, float(scale),
            int(bool(causal)), code, _stream_ptr()]
    if events is None:
        _check(lib.spark_mha_bwd(*args))
    else:
        _check(lib.spark_mha_bwd_marked(*args, events[0].slice_ptr(events[1])))
    return dQ, dK, dV


def spark_mha_bwd_static_max_rows() -> int:
    return int(load_library().spark_mha_bwd_static_max_rows())


def spark_mha_bwd_static(Q, K, V, O, LSE, dO, scale: float, causal: bool, dQ, dK, dV):
    """spark_mha_bwd without a workspace argument: the library's own fixed scratch array is used.
    The outputs must be passed in (the point of this entry point is that nothing is allocated)."""
    import torch
    lib = load_library()
    B, H, N, d = Q.shape
    for t, n in ((Q, "Q"), (K, "K"), (V, "V"), (O, "O"), (dO, "dO"), (dQ, "dQ"), (dK, "dK"), (dV, "dV")):
        _require(t, (B, H, N, d), Q.dtype, n)
    _require(LSE, (B, H, N), torch.float32, "LSE")
    _check(lib.spark_mha_bwd_static(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), LSE.data_ptr(),
                                    dO.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), B, H, N, d,
                                    float(scale), int(bool(causal)), _dtype_code(Q), _stream_ptr()))
    return dQ, dK, dV


def spark_layout_probe(dtype_code: int):
    """The 2304 floats of spark_layout_probe (see the header) as a device tensor."""
    import torch
    out = torch.full((2304,), float("nan"), dtype=torch.float32, device="cuda")
    _check(load_library().spark_layout_probe(out.data_ptr(), int(dtype_code), _stream_ptr()))
    return out


def spark_mha_bwd_atomic_workspace_bytes(B: int, H: int, Nq: int, Nk: int, d: int, dtype_code: int) -> int:
    return int(load_library().spark_mha_bwd_atomic_workspace_bytes(B, H, Nq, Nk, d, dtype_code))


def spark_mha_bwd_atomic(Q, K, V, O, LSE, dO, scale: float, causal: bool = False, dQ=None, dK=None,
                         dV=None, workspace=None):
    """The paper's own backward: one fused kernel, dQ accumulated in HBM with fp32 atomic adds."""
    import torch
    lib = load_library()
    B, H, Nq, d = Q.shape
    Nk = K.shape[2]
    for t, n in ((Q, "Q"), (O, "O"), (dO, "dO")):
        _require(t, (B, H, Nq, d), Q.dtype, n)
    for t, n in ((K, "K"), (V, "V")):
        _require(t, (B, H, Nk, d), Q.dtype, n)
    _require(LSE, (B, H, Nq), torch.float32, "LSE")
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(K) if dV is None else dV
    _require(dQ, (B, H, Nq, d), Q.dtype, "dQ")
    for t, n in ((dK, "dK"), (dV, "dV")):
        _require(t, (B, H, Nk, d), Q.dtype, n)
    code = _dtype_code(Q)
    need = spark_mha_bwd_atomic_workspace_bytes(B, H, Nq, Nk, d, code)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=Q.device)
    wbytes = workspace.numel() * workspace.element_size()
    _check(lib.spark_mha_bwd_atomic(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), LSE.data_ptr(),
                                    dO.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(),
                                    workspace.data_ptr(), wbytes, B, H, Nq, Nk, d, float(scale),
                                    int(bool(causal)), code, _stream_ptr()))
    return dQ, dK, dV
