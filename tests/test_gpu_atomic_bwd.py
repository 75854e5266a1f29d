"""The paper's own backward (Sec. 3.3: one fused kernel, dQ accumulated in HBM with fp32 atomic adds),
spark_mha_bwd_atomic, against the fp64 oracle to the same bar as the default backward; dK and dV
must be bitwise reproducible, dQ (whose adds arrive in any order: several results are correct) is
held to the tolerance only."""
import math

import numpy as np
import pytest

from paper_2502_12784_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _run(B, H, Nq, Nk, d, dtype, causal, seed, heads=None):
    import torch
    from paper_2502_12784_amd import spark_mha_bwd_atomic, spark_mha_cross_fwd
    scale = 1.0 / math.sqrt(d)
    inp = synth.make_inputs(B, H, Nq, d, dtype, seed, Nk=None if Nk == Nq else Nk)
    Q, K, V, dO = (pu.to_device(inp[n], dtype) for n in ("Q", "K", "V", "dO"))
    O, LSE = spark_mha_cross_fwd(Q, K, V, scale, causal)
    dQ, dK, dV = spark_mha_bwd_atomic(Q, K, V, O, LSE, dO, scale, causal)
    torch.cuda.synchronize()
    gpu = {"O": O, "LSE": LSE, "dQ": dQ, "dK": dK, "dV": dV}
    ref = pu.run_oracle(inp, dtype, scale, causal, heads=heads)
    m = pu.compare(gpu, ref, dtype, heads=heads)
    print(f"\n[atomic] B={B} H={H} Nq={Nq} Nk={Nk} d={d} {dtype} causal={causal}: {m}", flush=True)
    return m, (Q, K, V, O, LSE, dO, scale), gpu


SHAPES = [  # B, H, Nq, Nk, d
    (1, 2, 128, 128, 64), (2, 2, 256, 256, 128), (1, 3, 320, 320, 64), (1, 2, 63, 63, 128),
    (1, 2, 65, 65, 64), (1, 1, 777, 777, 128), (2, 1, 1, 1, 64), (1, 2, 200, 200, 72), (1, 1, 130, 130, 24),
]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("shape", SHAPES)
def test_atomic_backward_small_shapes(shape, dtype, causal):
    B, H, Nq, Nk, d = shape
    m, _, _ = _run(B, H, Nq, Nk, d, dtype, causal, seed=8800 + Nq + d)
    pu.assert_within_tolerance(m, (shape, dtype, causal))


@pytest.mark.parametrize("shape", [(1, 2, 100, 333, 64), (2, 1, 400, 96, 128), (1, 1, 1, 500, 64), (1, 2, 257, 1, 128)])
def test_atomic_backward_cross_lengths(shape):
    B, H, Nq, Nk, d = shape
    m, _, _ = _run(B, H, Nq, Nk, d, synth.BF16 if d == 128 else synth.F16, False, seed=8900 + Nq)
    pu.assert_within_tolerance(m, shape)


def test_atomic_backward_reproducibility_and_agreement_with_default():
    """dK, dV: no atomics, identical bits on every run.  dQ: close to the default backward's."""
    import torch
    from paper_2502_12784_amd import spark_mha_bwd_atomic, spark_mha_cross_bwd
    m, (Q, K, V, O, LSE, dO, scale), gpu = _run(2, 3, 1000, 1000, 128, synth.BF16, True, seed=8999)
    pu.assert_within_tolerance(m, "repro")
    again = spark_mha_bwd_atomic(Q, K, V, O, LSE, dO, scale, True)
    torch.cuda.synchronize()
    assert torch.equal(again[1], gpu["dK"]) and torch.equal(again[2], gpu["dV"])
    want = spark_mha_cross_bwd(Q, K, V, O, LSE, dO, scale, True)
    for a, b, n in zip((gpu["dQ"], gpu["dK"], gpu["dV"]), want, ("dQ", "dK", "dV")):
        rel = float((a.double() - b.double()).norm() / b.double().norm())
        assert rel <= 5e-3, (n, rel)


@pytest.mark.parametrize("name", ["C3", "C4"])
def test_atomic_backward_full_size_sampled_heads(name):
    w = synth.WORKLOADS[name]
    BH = w.B * w.H
    heads = [0, BH - 1]
    m, _, gpu = _run(w.B, w.H, w.N, w.N, w.d, w.dtype, w.causal, w.seed, heads=heads)
    pu.assert_within_tolerance(m, name)
    for n in ("dQ", "dK", "dV"):
        assert np.isfinite(pu.to_f64(gpu[n])).all(), n


def test_atomic_backward_workspace_is_checked():
    import torch
    import paper_2502_12784_amd as pkg
    need = pkg.spark_mha_bwd_atomic_workspace_bytes(2, 3, 100, 100, 64, 0)
    assert need == ((2 * 2 * 3 * 100 * 4 + 255) // 256) * 256 + 2 * 3 * 100 * 64 * 4
    Q = torch.zeros(2, 3, 100, 64, dtype=torch.float16, device="cuda")
    LSE = torch.zeros(2, 3, 100, dtype=torch.float32, device="cuda")
    ws = torch.empty(need - 1, dtype=torch.uint8, device="cuda")
    with pytest.raises(pkg.SparkError) as e:
        pkg.spark_mha_bwd_atomic(Q, Q, Q, Q, LSE, Q, 0.125, False, workspace=ws)
    assert e.value.status == -5
