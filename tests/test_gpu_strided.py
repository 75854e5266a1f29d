"""GPU tests of the strided entry points: the same kernels on [B,H,N,d] views with their own
batch / head / row strides (a permuted [B,N,H,d] projection output, slices of a packed QKV
buffer, padded rows).  Same arithmetic in the same order, so results must equal the contiguous
entry points bit for bit; one case is also checked against the oracle directly.
"""
import math

import pytest

from paper_2502_12784_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _contiguous_reference(Q, K, V, dO, scale, causal, dropout):
    from paper_2502_12784_amd import spark_mha_dropout_bwd, spark_mha_dropout_fwd
    p, seed, off = dropout
    Qc, Kc, Vc, dOc = (t.contiguous() for t in (Q, K, V, dO))
    O, LSE = spark_mha_dropout_fwd(Qc, Kc, Vc, scale, causal, p, seed, off)
    dQ, dK, dV = spark_mha_dropout_bwd(Qc, Kc, Vc, O, LSE, dOc, scale, causal, p, seed, off)
    return O, LSE, dQ, dK, dV


@pytest.mark.parametrize("dropout", [(0.0, 0, 0), (0.1, 77, 2)])
@pytest.mark.parametrize("shape,causal", [((2, 3, 200, 200, 64), True), ((1, 2, 130, 77, 128), False),
                                          ((2, 2, 333, 333, 128), True)])
def test_bnhd_views_equal_contiguous(shape, causal, dropout):
    """Q, K, V, dO stored [B,N,H,d] and viewed as [B,H,N,d]; outputs in the same layout."""
    import torch
    from paper_2502_12784_amd import spark_mha_strided_bwd, spark_mha_strided_fwd
    B, H, Nq, Nk, d = shape
    scale = 1.0 / math.sqrt(d)
    inp = synth.make_inputs(B, H, Nq, d, synth.F16, seed=500 + Nq + d, Nk=None if Nk == Nq else Nk)
    dev = {n: pu.to_device(inp[n], synth.F16) for n in ("Q", "K", "V", "dO")}
    # [B,H,N,d] values laid out as [B,N,H,d] memory
    Q, K, V, dO = (dev[n].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for n in ("Q", "K", "V", "dO"))
    assert not Q.is_contiguous() and Q.stride(1) == d and Q.stride(2) == H * d
    print(f"\n[strided] {shape} causal={causal} dropout={dropout}", flush=True)
    O, LSE = spark_mha_strided_fwd(Q, K, V, scale, causal, *dropout)
    assert O.stride() == Q.stride()
    dQ, dK, dV = spark_mha_strided_bwd(Q, K, V, O, LSE, dO, scale, causal, *dropout)
    torch.cuda.synchronize()
    ref = _contiguous_reference(Q, K, V, dO, scale, causal, dropout)
    for got, want, n in zip((O, LSE, dQ, dK, dV), ref, ("O", "LSE", "dQ", "dK", "dV")):
        assert torch.equal(got.contiguous(), want), n


def test_packed_qkv_buffer_and_padded_rows():
    """Q, K, V are slices of one [B,N,3,H,d] buffer, gradients go into another; O and dO have
    padded rows (row stride d + 8).  Checked against the contiguous path and the oracle."""
    import torch
    from paper_2502_12784_amd import spark_mha_strided_bwd, spark_mha_strided_fwd
    B, H, N, d = 2, 4, 257, 64
    scale = 0.125
    inp = synth.make_inputs(B, H, N, d, synth.BF16, seed=4321)
    dev = {n: pu.to_device(inp[n], synth.BF16) for n in ("Q", "K", "V", "dO")}
    qkv = torch.empty(B, N, 3, H, d, dtype=torch.bfloat16, device="cuda")
    for i, n in enumerate(("Q", "K", "V")):
        qkv[:, :, i] = dev[n].permute(0, 2, 1, 3)
    Q, K, V = (qkv[:, :, i].permute(0, 2, 1, 3) for i in range(3))
    assert Q.stride() == (N * 3 * H * d, d, 3 * H * d, 1)
    pad = torch.zeros(B, H, N, d + 8, dtype=torch.bfloat16, device="cuda")
    dO = pad[..., :d]
    dO.copy_(dev["dO"])
    Opad = torch.full((B, H, N, d + 8), 7.0, dtype=torch.bfloat16, device="cuda")
    O = Opad[..., :d]
    dqkv = torch.empty_like(qkv)
    dQ, dK, dV = (dqkv[:, :, i].permute(0, 2, 1, 3) for i in range(3))
    O, LSE = spark_mha_strided_fwd(Q, K, V, scale, True, O=O)
    spark_mha_strided_bwd(Q, K, V, O, LSE, dO, scale, True, dQ=dQ, dK=dK, dV=dV)
    torch.cuda.synchronize()
    assert Opad[..., d:].eq(7.0).all()  # the padding is untouched
    ref = _contiguous_reference(Q, K, V, dO, scale, True, (0.0, 0, 0))
    for got, want, n in zip((O, LSE, dQ, dK, dV), ref, ("O", "LSE", "dQ", "dK", "dV")):
        assert torch.equal(got.contiguous(), want), n
    gpu = {"O": O.contiguous(), "LSE": LSE, "dQ": dQ.contiguous(), "dK": dK.contiguous(), "dV": dV.contiguous()}
    m = pu.compare(gpu, pu.run_oracle(inp, synth.BF16, scale, True), synth.BF16)
    print(f"\n[strided] packed qkv: {m}", flush=True)
    pu.assert_within_tolerance(m, "packed qkv")


def test_bad_strides_are_refused():
    import torch
    from paper_2502_12784_amd import SparkError, spark_mha_strided_fwd
    x = torch.zeros(1, 2, 64, 72, dtype=torch.float16, device="cuda")
    Q = x[..., :64]
    bad = torch.zeros(1, 2, 64, 68, dtype=torch.float16, device="cuda")[..., :64]  # row stride 68: not 16-byte
    with pytest.raises(SparkError) as e:
        spark_mha_strided_fwd(bad, Q, Q, 0.125)
    assert e.value.status == -4
    with pytest.raises(ValueError):
        spark_mha_strided_fwd(Q.transpose(2, 3), Q, Q, 0.125)  # last dimension must be contiguous
