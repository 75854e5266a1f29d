"""C-ABI checks that need no GPU: the library loads, exports every symbol the header declares,
and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2502_12784_amd as pkg
from paper_2502_12784_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "spark_mha.h")

OK, E_NULL, E_SHAPE, E_DTYPE, E_ALIGN, E_WS, E_LAUNCH = 0, -1, -2, -3, -4, -5, -6


@pytest.fixture(scope="module")
def lib():
    return pkg.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spark_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_functions()
    assert set(names) == set(pkg.EXPORTS), (names, pkg.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    seen = set()
    for code in (OK, E_NULL, E_SHAPE, E_DTYPE, E_ALIGN, E_WS, E_LAUNCH, -99):
        s = pkg.status_str(code)
        assert isinstance(s, str) and s
        seen.add(s)
    assert len(seen) == 8


def _fwd(lib, q=0x1000, k=0x2000, v=0x3000, o=0x4000, lse=0x5000, B=1, H=1, N=128, d=64,
         scale=0.125, causal=0, dtype=0):
    return lib.spark_mha_fwd(q, k, v, o, lse, B, H, N, d, scale, causal, dtype, None)


def test_fwd_validation_has_no_side_effects(lib):
    # fake (never dereferenced) pointers: every call below must fail before any launch
    assert _fwd(lib, q=None) == E_NULL
    assert _fwd(lib, lse=None) == E_NULL
    assert _fwd(lib, B=0) == E_SHAPE
    assert _fwd(lib, N=0) == E_SHAPE
    assert _fwd(lib, d=100) == E_SHAPE
    assert _fwd(lib, d=136) == E_SHAPE
    assert _fwd(lib, scale=0.0) == E_SHAPE
    assert _fwd(lib, scale=-1.0) == E_SHAPE
    assert _fwd(lib, scale=float("nan")) == E_SHAPE
    assert _fwd(lib, scale=float("inf")) == E_SHAPE
    assert _fwd(lib, dtype=2) == E_DTYPE
    assert _fwd(lib, k=0x2008) == E_ALIGN
    assert _fwd(lib, B=1 << 20, H=1 << 10, N=1 << 12) == E_SHAPE  # grid would overflow
    assert _fwd(lib, N=1 << 25, d=128) == E_SHAPE                 # a head of 2 GiB or more
    for bad_d in (0, 4, 100, 136, 256):                           # multiples of 8 up to 128 only
        assert _fwd(lib, d=bad_d) == E_SHAPE


def _bwd(lib, fn="spark_mha_bwd", ws=0xA000, ws_bytes=1 << 20, dq=0x7000, B=1, H=1, N=128, d=64,
         scale=0.125, dtype=0, extra=()):
    f = getattr(lib, fn)
    return f(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, dq, 0x8000, 0x9000, ws, ws_bytes,
             B, H, N, d, scale, 0, dtype, None, *extra)


def test_bwd_validation(lib):
    assert _bwd(lib, dq=None) == E_NULL
    assert _bwd(lib, ws=None) == E_NULL
    assert _bwd(lib, d=100) == E_SHAPE
    assert _bwd(lib, dtype=7) == E_DTYPE
    assert _bwd(lib, dq=0x7004) == E_ALIGN
    need = pkg.spark_mha_bwd_workspace_bytes(1, 1, 128, 64, 0)
    assert need == 2 * 128 * 4
    assert _bwd(lib, ws_bytes=need - 1) == E_WS
    assert _bwd(lib, d=96, ws_bytes=need - 1) == E_WS  # d = 96 passes the shape checks
    assert _bwd(lib, d=8, ws_bytes=need - 1) == E_WS
    assert _bwd(lib, fn="spark_mha_bwd_marked", extra=(None,)) == E_NULL
    evs = (ctypes.c_void_p * 3)(1, None, 3)
    assert _bwd(lib, fn="spark_mha_bwd_marked", extra=(evs,)) == E_NULL


def test_static_workspace_entry_point_validation(lib):
    """spark_mha_bwd_static: refusals that happen before the device is touched."""
    def call(q=0x1000, B=1, H=1, N=128, d=64, dtype=0):
        return lib.spark_mha_bwd_static(q, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000, 0x8000, 0x9000,
                                        B, H, N, d, 0.125, 0, dtype, None)
    rows = pkg.spark_mha_bwd_static_max_rows()
    assert rows == 1 << 20
    assert call(q=None) == E_NULL
    assert call(d=100) == E_SHAPE
    assert call(dtype=3) == E_DTYPE
    assert call(B=2, H=8, N=(rows // 16) + 1) == E_WS   # one row too many for the fixed scratch array


def test_atomic_backward_validation(lib):
    """spark_mha_bwd_atomic: same refusals as the default backward, and its own workspace size."""
    def call(ws=0xA000, ws_bytes=1 << 30, dq=0x7000, Nq=128, Nk=96, d=64, causal=0, dtype=0):
        return lib.spark_mha_bwd_atomic(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, dq, 0x8000, 0x9000,
                                        ws, ws_bytes, 1, 2, Nq, Nk, d, 0.125, causal, dtype, None)
    need = pkg.spark_mha_bwd_atomic_workspace_bytes(1, 2, 128, 96, 64, 0)
    assert need == 2 * 2 * 128 * 4 + 2 * 128 * 64 * 4   # statistics (already a multiple of 256) + fp32 dQ
    assert pkg.spark_mha_bwd_atomic_workspace_bytes(1, 2, 100, 96, 64, 0) == 1792 + 2 * 100 * 64 * 4  # padded to 256
    assert pkg.spark_mha_bwd_atomic_workspace_bytes(1, 2, 128, 96, 100, 0) == 0
    assert call(ws=None) == E_NULL
    assert call(dq=None) == E_NULL
    assert call(d=100) == E_SHAPE
    assert call(causal=1) == E_SHAPE            # causal needs Nq == Nk
    assert call(dtype=9) == E_DTYPE
    assert call(dq=0x7008) == E_ALIGN
    assert call(ws_bytes=need - 1) == E_WS


def test_dropout_marked_validation(lib):
    def call(events, p=0.1):
        return lib.spark_mha_dropout_bwd_marked(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000, 0x8000,
                                                0x9000, 0xA000, 1 << 20, 1, 1, 128, 128, 64, 0.125, 0, p, 1234, 0,
                                                0, None, events)
    assert call(None) == E_NULL
    assert call((ctypes.c_void_p * 3)(1, 2, None)) == E_NULL
    assert call((ctypes.c_void_p * 3)(1, 2, 3), p=1.5) == E_SHAPE


def test_cross_validation(lib):
    def fwd(Nq=128, Nk=96, causal=0, **kw):
        a = dict(q=0x1000, k=0x2000, v=0x3000, o=0x4000, lse=0x5000, B=1, H=1, d=64, scale=0.125, dtype=0)
        a.update(kw)
        return lib.spark_mha_cross_fwd(a["q"], a["k"], a["v"], a["o"], a["lse"], a["B"], a["H"], Nq, Nk,
                                       a["d"], a["scale"], causal, a["dtype"], None)

    def bwd(Nq=128, Nk=96, causal=0, ws_bytes=1 << 20, dk=0x8000):
        return lib.spark_mha_cross_bwd(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000, dk, 0x9000,
                                       0xA000, ws_bytes, 1, 1, Nq, Nk, 64, 0.125, causal, 0, None)

    assert fwd(Nq=0) == E_SHAPE
    assert fwd(Nk=0) == E_SHAPE
    assert fwd(causal=1) == E_SHAPE               # causal needs Nq == Nk
    assert fwd(Nk=1 << 25, d=128) == E_SHAPE      # Nk*d >= 2^31
    assert fwd(v=None) == E_NULL
    assert fwd(o=0x4002) == E_ALIGN
    assert fwd(dtype=5) == E_DTYPE
    assert bwd(causal=1) == E_SHAPE
    assert bwd(Nk=0) == E_SHAPE
    assert bwd(dk=None) == E_NULL
    need = pkg.spark_mha_cross_bwd_workspace_bytes(1, 1, 128, 96, 64, 0)
    assert need == 2 * 128 * 4                    # sized by the queries, not the keys
    assert bwd(ws_bytes=need - 1) == E_WS
    assert pkg.spark_mha_cross_bwd_workspace_bytes(1, 1, 128, 0, 64, 0) == 0


def test_dropout_validation(lib):
    assert pkg.spark_dropout_threshold(0.1) == 26      # the paper's rate, realised to 8 bits
    assert pkg.spark_dropout_threshold(0.0) == 0
    assert pkg.spark_dropout_threshold(255.4 / 256) == 255
    assert pkg.spark_dropout_threshold(255.6 / 256) == -1
    assert pkg.spark_dropout_threshold(-1e-3) == -1
    assert pkg.spark_dropout_threshold(float("nan")) == -1

    def fwd(p=0.1, q=0x1000, Nq=128, Nk=128, causal=0):
        return lib.spark_mha_dropout_fwd(q, 0x2000, 0x3000, 0x4000, 0x5000, 1, 1, Nq, Nk, 64, 0.125, causal,
                                         p, 1234, 0, 0, None)

    def bwd(p=0.1, ws_bytes=1 << 20, Nk=128):
        return lib.spark_mha_dropout_bwd(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000, 0x8000,
                                         0x9000, 0xA000, ws_bytes, 1, 1, 128, Nk, 64, 0.125, 0, p, 1234, 0,
                                         0, None)

    assert fwd(p=1.0) == E_SHAPE
    assert fwd(p=-0.1) == E_SHAPE
    assert fwd(q=None) == E_NULL
    assert fwd(Nk=64, causal=1) == E_SHAPE
    assert bwd(p=float("nan")) == E_SHAPE
    assert bwd(ws_bytes=8) == E_WS
    assert bwd(Nk=0) == E_SHAPE
    assert lib.spark_dropout_mask(None, 1, 1, 4, 4, 0.1, 1, 0, None) == E_NULL
    assert lib.spark_dropout_mask(0x1000, 1, 1, 0, 4, 0.1, 1, 0, None) == E_SHAPE
    assert lib.spark_dropout_mask(0x1000, 1, 1, 4, 4, 2.0, 1, 0, None) == E_SHAPE


def test_strided_validation(lib):
    S = pkg.Strides

    def fwd(sq=S(128 * 64, 64 * 128, 64), so=S(128 * 64, 64 * 128, 64), sk=S(128 * 64, 64 * 128, 64), N=128, d=64):
        return lib.spark_mha_strided_fwd(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, sq, sk, sk, so, 1, 1, N, N,
                                         d, 0.125, 0, 0.0, 0, 0, 0, None)

    assert fwd(sq=None) == E_NULL
    assert fwd(sq=S(0, 0, 32)) == E_SHAPE              # rows would overlap: row stride < d
    assert fwd(sq=S(-8, 0, 64)) == E_SHAPE
    assert fwd(sk=S(0, 0, 68)) == E_ALIGN              # 136-byte rows
    assert fwd(so=S(4, 0, 64)) == E_ALIGN
    assert fwd(sq=S(0, 0, 1 << 24), N=1024) == E_SHAPE  # one head would span 2 GiB or more
    # a zero batch / head stride broadcasts an input, but would make every (batch, head) of an
    # output store to the same rows
    def fwd_bh(B, H, so, sq=S(0, 0, 64)):
        return lib.spark_mha_strided_fwd(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, sq, sq, sq, so, B, H, 128,
                                         128, 64, 0.125, 0, 0.0, 0, 0, 0, None)
    assert fwd_bh(2, 1, S(0, 128 * 64, 64)) == E_SHAPE
    assert fwd_bh(1, 2, S(2 * 128 * 64, 0, 64)) == E_SHAPE
    eight = [S(128 * 64, 64 * 128, 64)] * 8
    args = [0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000, 0x8000, 0x9000]
    tail = [0xA000, 1 << 20, 1, 1, 128, 128, 64, 0.125, 0, 0.0, 0, 0, 0, None]
    assert lib.spark_mha_strided_bwd(*args, *eight[:7], None, *tail) == E_NULL
    assert lib.spark_mha_strided_bwd(*args, *eight[:7], S(0, 0, 8), *tail) == E_SHAPE
    tail2 = [0xA000, 1 << 20, 2, 2, 128, 128, 64, 0.125, 0, 0.0, 0, 0, 0, None]
    good = S(2 * 128 * 64, 128 * 64, 64)
    for pos in (5, 6, 7):  # dQ, dK, dV
        for zero in (S(0, 128 * 64, 64), S(2 * 128 * 64, 0, 64)):
            st = [good] * 8
            st[pos] = zero
            assert lib.spark_mha_strided_bwd(*args, *st, *tail2) == E_SHAPE
    tail[1] = 8
    assert lib.spark_mha_strided_bwd(*args, *eight, *tail) == E_WS


def test_workspace_bytes(lib):
    assert pkg.spark_mha_bwd_workspace_bytes(4, 16, 4096, 128, 1) == 2 * 4 * 16 * 4096 * 4
    assert pkg.spark_mha_bwd_workspace_bytes(4, 16, 4096, 100, 1) == 0
    assert pkg.spark_mha_bwd_workspace_bytes(0, 16, 4096, 128, 1) == 0


def test_binding_refuses_host_tensors():
    import torch
    x = torch.zeros(1, 1, 8, 64, dtype=torch.float16)
    with pytest.raises(ValueError):
        pkg.spark_mha_fwd(x, x, x, 0.125, False)


def test_product_does_not_import_oracle():
    """The product package must not reach into oracle/ (parity would be void)."""
    pkgdir = os.path.join(ROOT, "paper_2502_12784_amd")
    for dirpath, _, files in os.walk(pkgdir):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle|#include\s*[<\"].*oracle", text, flags=re.M), f
                assert "liboracle" not in text and "mha_oracle" not in text, f
