"""ctypes front end of the fp64 C oracle in ``mha_oracle.c``.

TEST INFRASTRUCTURE ONLY: the HIP path never imports or calls this module, and
this module imports nothing from the HIP package.  All arithmetic lives in the C
file; this wrapper only checks shapes, widens nothing and converts nothing
(inputs must already be float64 arrays: Q and dO of shape [B, H, Nq, d], K and V
of shape [B, H, Nk, d]; self-attention has Nq = Nk, the cross-attention of the
decoder's second attention layer in Sec. 2.1 does not).

The definitions follow the paper's Eq. 1 (forward), Sec. 3.2.1 Eq. 2 (softmax,
with l = sum of f) and Sec. 3.3 Eq. 4 (backward, dK = dS^T Q); dropout (Sec. 4.1,
4.2) acts on P through an explicit keep mask, which ``dropout_mask`` draws with
Philox4x32-10.  See the header of ``mha_oracle.c`` for the formulas and the
readings taken.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mha_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_mha.so")
_default = None

_dp = ctypes.POINTER(ctypes.c_double)
_u8p = ctypes.POINTER(ctypes.c_ubyte)
_u32p = ctypes.POINTER(ctypes.c_uint32)
GCC_FLAGS = ["-O3", "-mavx2", "-mfma", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra"]


def compile_source(src: str, out: str) -> str:
    """gcc one C source into a shared library (plain -O3, AVX2; no fast-math)."""
    tmp = out + ".tmp.%d" % os.getpid()
    subprocess.run(["gcc"] + GCC_FLAGS + ["-o", tmp, src, "-lm"], check=True)
    os.replace(tmp, out)
    return out


def build(force: bool = False) -> str:
    """Compile the C oracle next to its source if it is missing or stale."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_source(_SRC, _LIB)
    return _LIB


def _chk(Q, K, V, dO=None):
    """Shapes: Q (and dO) [B,H,Nq,d]; K, V [B,H,Nk,d]."""
    if Q.ndim != 4 or K.ndim != 4:
        raise ValueError("expected [B, H, N, d] arrays")
    if K.shape[:2] != Q.shape[:2] or K.shape[3] != Q.shape[3] or V.shape != K.shape:
        raise ValueError("K, V must be [B, H, Nk, d] with Q's B, H, d")
    if dO is not None and dO.shape != Q.shape:
        raise ValueError("dO must have Q's shape")
    arrs = [a for a in (Q, K, V, dO) if a is not None]
    for a in arrs:
        if a.dtype != np.float64:
            raise ValueError("oracle inputs must be float64 arrays")
    return [np.ascontiguousarray(a) for a in arrs]


def _p(a):
    return a.ctypes.data_as(_dp) if a is not None else None


class OracleLib:
    """The oracle's entry points bound to one shared library (the default build, or a
    library a test compiled itself, e.g. from a deliberately broken copy of the source)."""

    def __init__(self, path: str):
        lib = ctypes.CDLL(path)
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_mha_fwd.restype = ctypes.c_int
        lib.oracle_mha_fwd.argtypes = [_dp, _dp, _dp, _dp, _dp, _dp, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_int,
                                       _u8p, ctypes.c_double]
        lib.oracle_mha_bwd.restype = ctypes.c_int
        lib.oracle_mha_bwd.argtypes = [_dp] * 10 + [ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                    ctypes.c_int, ctypes.c_double, ctypes.c_int,
                                                    _u8p, ctypes.c_double]
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
        lib.oracle_dropout_mask.restype = ctypes.c_int
        lib.oracle_dropout_mask.argtypes = [_u8p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                            ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int]
        self._lib = lib

    def num_threads(self) -> int:
        """OpenMP threads the oracle will use."""
        return int(self._lib.oracle_num_threads())

    def philox4x32_10(self, ctr, key):
        """The four 32-bit output words of Philox4x32-10 for a 4-word counter, 2-word key."""
        c = (ctypes.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
        k = (ctypes.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
        out = (ctypes.c_uint32 * 4)()
        self._lib.oracle_philox4x32_10(c, k, out)
        return [int(x) for x in out]

    def dropout_mask(self, B: int, H: int, Nq: int, Nk: int, seed: int, offset: int,
                     threshold: int) -> np.ndarray:
        """Keep mask [B,H,Nq,Nk] uint8 (1 = keep); an entry is dropped with probability
        threshold/256."""
        M = np.empty((B, H, Nq, Nk), dtype=np.uint8)
        rc = self._lib.oracle_dropout_mask(M.ctypes.data_as(_u8p), B * H, Nq, Nk, int(seed),
                                           int(offset), int(threshold))
        if rc != 0:
            raise RuntimeError("oracle_dropout_mask failed (%d)" % rc)
        return M

    @staticmethod
    def _keep_arg(keep, shape):
        if keep is None:
            return None, None
        if keep.dtype != np.uint8 or keep.shape != shape:
            raise ValueError("keep must be a uint8 array of shape %s" % (shape,))
        keep = np.ascontiguousarray(keep)
        return keep, keep.ctypes.data_as(_u8p)

    def mha_fwd(self, Q, K, V, scale: float, causal: bool, return_P: bool = False, keep=None,
                keep_scale: float = 1.0):
        """O [B,H,Nq,d], LSE [B,H,Nq] (and P [B,H,Nq,Nk] if asked) in float64.
        keep: optional dropout keep mask [B,H,Nq,Nk] uint8; survivors are scaled by keep_scale."""
        Q, K, V = _chk(Q, K, V)
        B, H, Nq, d = Q.shape
        Nk = K.shape[2]
        keep, keep_p = self._keep_arg(keep, (B, H, Nq, Nk))
        O = np.empty_like(Q)
        LSE = np.empty((B, H, Nq), dtype=np.float64)
        P = np.empty((B, H, Nq, Nk), dtype=np.float64) if return_P else None
        rc = self._lib.oracle_mha_fwd(_p(Q), _p(K), _p(V), _p(O), _p(LSE), _p(P), B * H, Nq, Nk, d,
                                      float(scale), int(bool(causal)), keep_p, float(keep_scale))
        if rc != 0:
            raise RuntimeError("oracle_mha_fwd failed (%d)" % rc)
        return (O, LSE, P) if return_P else (O, LSE)

    def mha_bwd(self, Q, K, V, dO, scale: float, causal: bool, keep=None, keep_scale: float = 1.0):
        """dict with dQ [B,H,Nq,d], dK, dV [B,H,Nk,d], and the oracle's own O, LSE, D."""
        Q, K, V, dO = _chk(Q, K, V, dO)
        B, H, Nq, d = Q.shape
        Nk = K.shape[2]
        keep, keep_p = self._keep_arg(keep, (B, H, Nq, Nk))
        dQ, O = np.empty_like(Q), np.empty_like(Q)
        dK, dV = np.empty_like(K), np.empty_like(K)
        LSE = np.empty((B, H, Nq), dtype=np.float64)
        D = np.empty((B, H, Nq), dtype=np.float64)
        rc = self._lib.oracle_mha_bwd(_p(Q), _p(K), _p(V), _p(dO), _p(dQ), _p(dK), _p(dV), _p(O),
                                      _p(LSE), _p(D), B * H, Nq, Nk, d, float(scale),
                                      int(bool(causal)), keep_p, float(keep_scale))
        if rc != 0:
            raise RuntimeError("oracle_mha_bwd failed (%d)" % rc)
        return {"dQ": dQ, "dK": dK, "dV": dV, "O": O, "LSE": LSE, "D": D}


def default() -> OracleLib:
    global _default
    if _default is None:
        _default = OracleLib(build())
    return _default


def num_threads() -> int:
    return default().num_threads()


def mha_fwd(Q, K, V, scale: float, causal: bool, return_P: bool = False, keep=None,
            keep_scale: float = 1.0):
    return default().mha_fwd(Q, K, V, scale, causal, return_P, keep, keep_scale)


def mha_bwd(Q, K, V, dO, scale: float, causal: bool, keep=None, keep_scale: float = 1.0):
    return default().mha_bwd(Q, K, V, dO, scale, causal, keep, keep_scale)


def philox4x32_10(ctr, key):
    return default().philox4x32_10(ctr, key)


def dropout_mask(B, H, Nq, Nk, seed, offset, threshold):
    return default().dropout_mask(B, H, Nq, Nk, seed, offset, threshold)
