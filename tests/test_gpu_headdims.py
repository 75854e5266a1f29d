"""GPU parity for head dimensions other than the paper's 64 and 128 (Sec. 4.1 measures those
two only): every multiple of 8 up to 128 runs in the kernel built for the next wider row, with
the missing columns read as zeros and never stored.  Same bar as the other parity tests, all
elements against the fp64 oracle; plus a check that nothing beyond column d is written when the
rows of the output are padded.
"""
import math

import numpy as np
import pytest

from paper_2502_12784_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

SEED = 0x9E3779B97F4A7C15
DIMS = [8, 16, 24, 32, 40, 48, 56, 72, 80, 96, 104, 112, 120]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("d", DIMS)
def test_head_dim_all_elements(d, dtype, causal):
    """N = 200 spans several tiles of every kernel and leaves a ragged tail."""
    B, H, N = 1, 2, 200
    scale = 1.0 / math.sqrt(d)
    inp = synth.make_inputs(B, H, N, d, dtype, seed=9000 + d)
    print(f"\n[headdim] d={d} {dtype} causal={causal}", flush=True)
    gpu = pu.run_gpu(inp, dtype, scale, causal)
    ref = pu.run_oracle(inp, dtype, scale, causal)
    m = pu.compare(gpu, ref, dtype)
    print(f"[headdim] d={d} {dtype} causal={causal}: {m}", flush=True)
    pu.assert_within_tolerance(m, (d, dtype, causal))


@pytest.mark.parametrize("d,Nq,Nk", [(40, 150, 333), (96, 333, 150), (24, 1, 70), (120, 70, 1)])
def test_head_dim_cross_attention(d, Nq, Nk):
    scale = 1.0 / math.sqrt(d)
    inp = synth.make_inputs(2, 2, Nq, d, synth.BF16, seed=9100 + d, Nk=Nk)
    print(f"\n[headdim] cross d={d} Nq={Nq} Nk={Nk}", flush=True)
    gpu = pu.run_gpu(inp, synth.BF16, scale, False)
    ref = pu.run_oracle(inp, synth.BF16, scale, False)
    m = pu.compare(gpu, ref, synth.BF16)
    print(f"[headdim] cross d={d}: {m}", flush=True)
    pu.assert_within_tolerance(m, ("cross", d))


@pytest.mark.parametrize("d,causal", [(32, True), (80, False), (104, True)])
def test_head_dim_with_dropout(d, causal):
    from paper_2502_12784_amd import spark_dropout_threshold
    scale = 1.0 / math.sqrt(d)
    inp = synth.make_inputs(1, 2, 260, d, synth.F16, seed=9200 + d)
    print(f"\n[headdim] dropout d={d} causal={causal}", flush=True)
    gpu = pu.run_gpu(inp, synth.F16, scale, causal, dropout=(0.1, SEED, 3))
    ref = pu.run_oracle(inp, synth.F16, scale, causal, dropout=(spark_dropout_threshold(0.1), SEED, 3))
    m = pu.compare(gpu, ref, synth.F16)
    print(f"[headdim] dropout d={d}: {m}", flush=True)
    pu.assert_within_tolerance(m, ("dropout", d))


@pytest.mark.parametrize("d", [40, 96])
def test_head_dim_strided_rows_leave_the_padding_alone(d):
    """[B,N,H,d] tensors with rows padded to 128 elements: results equal the contiguous entry
    points bit for bit, and the padding of every output row keeps the value it had."""
    import torch
    from paper_2502_12784_amd import (spark_mha_bwd, spark_mha_fwd, spark_mha_strided_bwd,
                                      spark_mha_strided_fwd)
    B, H, N, row = 2, 3, 170, 128
    scale = 1.0 / math.sqrt(d)
    inp = synth.make_inputs(B, H, N, d, synth.BF16, seed=9300 + d)
    dev = {n: pu.to_device(inp[n], synth.BF16) for n in ("Q", "K", "V", "dO")}

    def padded(t=None):
        buf = torch.full((B, N, H, row), 7.0, dtype=torch.bfloat16, device="cuda")
        view = buf[..., :d].permute(0, 2, 1, 3)  # [B,H,N,d], row stride H*row, head stride row
        if t is not None:
            view.copy_(t)
        return buf, view

    (_, Q), (_, K), (_, V), (_, dO) = (padded(dev[n]) for n in ("Q", "K", "V", "dO"))
    (Ob, O), (dQb, dQ), (dKb, dK), (dVb, dV) = (padded() for _ in range(4))
    print(f"\n[headdim] strided d={d}", flush=True)
    _, LSE = spark_mha_strided_fwd(Q, K, V, scale, True, 0.0, 0, 0, O=O)
    spark_mha_strided_bwd(Q, K, V, O, LSE, dO, scale, True, 0.0, 0, 0, dQ=dQ, dK=dK, dV=dV)
    Oc, LSEc = spark_mha_fwd(dev["Q"], dev["K"], dev["V"], scale, True)
    ref = spark_mha_bwd(dev["Q"], dev["K"], dev["V"], Oc, LSEc, dev["dO"], scale, True)
    torch.cuda.synchronize()
    assert torch.equal(LSE, LSEc)
    for got, want, n in zip((O, dQ, dK, dV), (Oc,) + tuple(ref), ("O", "dQ", "dK", "dV")):
        assert torch.equal(got.contiguous(), want), n
    for buf, n in ((Ob, "O"), (dQb, "dQ"), (dKb, "dK"), (dVb, "dV")):
        assert bool((buf[..., d:] == 7.0).all()), n + ": columns beyond d were written"


def test_head_dim_not_a_multiple_of_8_is_refused():
    import torch
    from paper_2502_12784_amd import SparkError, spark_mha_fwd
    for d in (4, 100, 136):
        Q = torch.zeros((1, 1, 16, d), dtype=torch.float16, device="cuda")
        with pytest.raises(SparkError):
            spark_mha_fwd(Q, Q.clone(), Q.clone(), 0.1, False)
