"""GPU parity for cross-attention (Nq queries, Nk keys/values; paper Sec. 2.1, the decoder's
second attention layer) through spark_mha_cross_fwd / spark_mha_cross_bwd against the fp64
oracle.  Same bar as the self-attention tests.  Non-causal only: the mask needs Nq == Nk.
"""
import math

import numpy as np
import pytest

from paper_2502_12784_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

# (B, H, Nq, Nk, d): fewer queries than keys and the reverse, single rows, ragged tails on
# either side, several tiles on either side
SHAPES = [
    (1, 2, 200, 77, 64), (2, 3, 77, 200, 64), (1, 2, 1, 300, 64), (1, 2, 300, 1, 64),
    (1, 2, 129, 257, 64), (1, 1, 640, 128, 64),
    (1, 2, 200, 77, 128), (2, 2, 77, 200, 128), (1, 2, 1, 300, 128), (1, 2, 300, 1, 128),
    (1, 2, 129, 257, 128), (1, 1, 128, 640, 128),
]


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("shape", SHAPES)
def test_cross_small_shapes_all_elements(shape, dtype):
    B, H, Nq, Nk, d = shape
    scale = 1.0 / math.sqrt(d)
    inp = synth.make_inputs(B, H, Nq, d, dtype, seed=8000 + Nq + 3 * Nk + d, Nk=Nk)
    assert inp["K"].shape == (B, H, Nk, d) and inp["Q"].shape == (B, H, Nq, d)
    print(f"\n[cross] {shape} {dtype}", flush=True)
    gpu = pu.run_gpu(inp, dtype, scale, False)
    assert tuple(gpu["dK"].shape) == (B, H, Nk, d) and tuple(gpu["dQ"].shape) == (B, H, Nq, d)
    ref = pu.run_oracle(inp, dtype, scale, False)
    m = pu.compare(gpu, ref, dtype)
    print(f"[cross] {shape} {dtype}: {m}", flush=True)
    pu.assert_within_tolerance(m, (shape, dtype))


def test_cross_equals_self_entry_point_when_lengths_match():
    """With Nq == Nk the cross entry points are the self-attention ones, bit for bit, causal too."""
    import torch
    from paper_2502_12784_amd import (spark_mha_bwd, spark_mha_cross_bwd, spark_mha_cross_fwd,
                                      spark_mha_fwd)
    inp = synth.make_inputs(1, 3, 333, 128, synth.BF16, seed=31)
    Q, K, V, dO = (pu.to_device(inp[n], synth.BF16) for n in ("Q", "K", "V", "dO"))
    for causal in (False, True):
        O1, L1 = spark_mha_fwd(Q, K, V, 0.1, causal)
        O2, L2 = spark_mha_cross_fwd(Q, K, V, 0.1, causal)
        g1 = spark_mha_bwd(Q, K, V, O1, L1, dO, 0.1, causal)
        g2 = spark_mha_cross_bwd(Q, K, V, O2, L2, dO, 0.1, causal)
        torch.cuda.synchronize()
        assert torch.equal(O1, O2) and torch.equal(L1, L2)
        for a, b in zip(g1, g2):
            assert torch.equal(a, b)


def test_cross_causal_with_unequal_lengths_is_refused():
    import torch
    from paper_2502_12784_amd import SparkError, spark_mha_cross_fwd
    Q = torch.zeros(1, 1, 64, 64, dtype=torch.float16, device="cuda")
    K = torch.zeros(1, 1, 96, 64, dtype=torch.float16, device="cuda")
    with pytest.raises(SparkError) as e:
        spark_mha_cross_fwd(Q, K, K, 0.125, True)
    assert e.value.status == -2


@pytest.mark.parametrize("Nq,Nk,d,dtype", [(1024, 4096, 128, synth.BF16), (4096, 512, 64, synth.F16)])
def test_cross_training_size_sampled_heads(Nq, Nk, d, dtype):
    """A decoder-sized problem (B = 4, H = 16): full-size GPU run, two heads checked in full,
    sum invariants on every head."""
    B, H = 4, 16
    scale = 1.0 / math.sqrt(d)
    inp = synth.make_inputs(B, H, Nq, d, dtype, seed=9000 + Nq + Nk, Nk=Nk)
    gpu = pu.run_gpu(inp, dtype, scale, False)
    heads = [0, B * H - 1]
    ref = pu.run_oracle(inp, dtype, scale, False, heads=heads)
    m = pu.compare(gpu, ref, dtype, heads=heads)
    print(f"\n[cross] Nq={Nq} Nk={Nk} d={d} {dtype} heads={heads}: {m}", flush=True)
    pu.assert_within_tolerance(m, (Nq, Nk, d, dtype))
    dK = pu.to_f64(gpu["dK"]); dV = pu.to_f64(gpu["dV"])
    dO = synth.bits_to_f64(inp["dO"], dtype)
    assert np.abs(dK.sum(2)).max() <= 2e-2 * np.abs(dK).sum(2).max()
    assert np.abs(dV.sum(2) - dO.sum(2)).max() <= 2e-2 * np.abs(dO).sum(2).max()
    for n in ("O", "LSE", "dQ", "dK", "dV"):
        assert np.isfinite(pu.to_f64(gpu[n])).all(), n
