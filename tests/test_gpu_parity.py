"""GPU parity: HIP path (through the C ABI) against the fp64 CPU oracle, same seeded inputs.

Bar (tests/parity_util.py): fp16: |O - O_ref| <= 2e-3 + half an output ulp at |O_ref| (the output
is rounded once to 16 bits), and raw |O - O_ref| <= 2e-3 on the fp16 benchmark configurations;
bf16: the same, except that elements which exceed it must lie within the bound u * P|V| on what
rounding P to the bf16 operand type can do (their number is printed); |LSE - LSE_ref| <= 2e-3;
relative L2 error <= 1e-2 for each of dQ, dK, dV, and every single row of them within 2e-2 (fp16) /
5e-2 (bf16) of its own norm plus twice the typical row norm, so that one wrong row cannot hide in
a whole-tensor norm.
"""
import math

import numpy as np
import pytest

from paper_2502_12784_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _run_full(B, H, N, d, dtype, causal, seed, sigma_qk=1.0, scale=None):
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    inp = synth.make_inputs(B, H, N, d, dtype, seed, sigma_qk=sigma_qk)
    gpu = pu.run_gpu(inp, dtype, scale, causal)
    ref = pu.run_oracle(inp, dtype, scale, causal)
    m = pu.compare(gpu, ref, dtype)
    print(f"\n[parity] B={B} H={H} N={N} d={d} {dtype} causal={causal}: {m}", flush=True)
    return m


# Small shapes, every head checked element by element: several tiles, ragged tails,
# both head dims, both dtypes, both mask settings.
SMALL = [
    (1, 2, 128, 64), (2, 2, 256, 128), (1, 3, 320, 64), (1, 2, 384, 128),
    (2, 1, 1, 64), (1, 2, 63, 128), (1, 2, 65, 64), (1, 1, 200, 128), (1, 2, 333, 64),
    (1, 1, 777, 128),
]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
@pytest.mark.parametrize("shape", SMALL)
def test_small_shapes_all_elements(shape, dtype, causal):
    B, H, N, d = shape
    m = _run_full(B, H, N, d, dtype, causal, seed=7000 + N + d)
    pu.assert_within_tolerance(m, (shape, dtype, causal))


def test_config_C1_full():
    w = synth.WORKLOADS["C1"]
    m = _run_full(w.B, w.H, w.N, w.d, w.dtype, w.causal, w.seed, w.sigma_qk)
    pu.assert_within_tolerance(m, "C1")
    assert m["O_maxabs"] <= pu.TOL_ABS, m  # fp16: the stated bound holds without any allowance


def test_wide_logits_small():
    """Logits with std 3 (the long-sequence config's distribution) at a size checked in full."""
    m = _run_full(1, 2, 512, 64, synth.F16, False, seed=4242, sigma_qk=math.sqrt(3.0))
    pu.assert_within_tolerance(m, "wide logits")


@pytest.mark.parametrize("name", ["C2", "C3", "C4", "C5"])
def test_full_size_configs_sampled_heads(name):
    """Full-size run in the benchmark's launch configuration; the oracle checks the first,
    a middle and the last (batch, head) element by element."""
    w = synth.WORKLOADS[name]
    inp = synth.make_workload_inputs(w)
    gpu = pu.run_gpu(inp, w.dtype, w.scale, w.causal)
    BH = w.B * w.H
    heads = sorted({0, BH // 2 + 1, BH - 1}) if w.N <= 4096 else [0, BH - 1]
    ref = pu.run_oracle(inp, w.dtype, w.scale, w.causal, heads=heads)
    m = pu.compare(gpu, ref, w.dtype, heads=heads)
    print(f"\n[parity] {name} heads={heads}: {m}", flush=True)
    pu.assert_within_tolerance(m, name)
    if w.dtype == synth.F16:
        assert m["O_maxabs"] <= pu.TOL_ABS, m  # fp16: the stated bound holds without any allowance
    # properties that hold at any size, checked on every head of the GPU result
    dK = pu.to_f64(gpu["dK"]); dV = pu.to_f64(gpu["dV"])
    dO = synth.bits_to_f64(inp["dO"], w.dtype)
    # columns of dK sum to zero over keys; sum_j dV_j = sum_i dO_i (rows of P sum to one)
    scale_k = np.abs(dK).sum(2).max()
    assert np.abs(dK.sum(2)).max() <= 2e-2 * scale_k
    assert np.abs(dV.sum(2) - dO.sum(2)).max() <= 2e-2 * np.abs(dO).sum(2).max()
    for n in ("O", "LSE", "dQ", "dK", "dV"):
        assert np.isfinite(pu.to_f64(gpu[n])).all(), n


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_many_heads_ragged_wide_workgroups(dtype, causal):
    """Enough (batch, head) pairs at d = 128 for the forward to pick its 256-query workgroups, with a
    sequence length that is a multiple of neither 256 nor 64; sampled heads against the oracle."""
    B, H, N, d = 8, 16, 2100, 128  # the 256-query workgroups are chosen from 2048 keys on
    inp = synth.make_inputs(B, H, N, d, dtype, seed=600 + int(causal))
    scale = 1.0 / math.sqrt(d)
    gpu = pu.run_gpu(inp, dtype, scale, causal)
    heads = [0, 77, B * H - 1]
    ref = pu.run_oracle(inp, dtype, scale, causal, heads=heads)
    m = pu.compare(gpu, ref, dtype, heads=heads)
    print(f"\n[parity] wide workgroups N={N} {dtype} causal={causal}: {m}", flush=True)
    pu.assert_within_tolerance(m, ("wide", dtype, causal))
    for n in ("O", "LSE", "dQ", "dK", "dV"):
        assert np.isfinite(pu.to_f64(gpu[n])).all(), n


def test_bitwise_reproducible():
    """No atomics anywhere: two runs give identical bits."""
    import torch
    w = synth.WORKLOADS["C3"]
    inp = synth.make_inputs(2, 2, w.N, w.d, w.dtype, 99)
    a = pu.run_gpu(inp, w.dtype, w.scale, True)
    b = pu.run_gpu(inp, w.dtype, w.scale, True)
    for n in ("O", "LSE", "dQ", "dK", "dV"):
        assert torch.equal(a[n], b[n]), n


@pytest.mark.parametrize("d,causal", [(64, True), (128, False)])
def test_paper_sweep_longest_sequence_sampled(d, causal):
    """The longest point of the paper's own grid (Sec. 4.1): N = 16384, B = 1, H = 2048/d, fp16.
    Full-size GPU run; the oracle checks one (batch, head) element by element."""
    N, B, H = 16384, 1, 2048 // d
    inp = synth.make_inputs(B, H, N, d, synth.F16, seed=16384 + d)
    gpu = pu.run_gpu(inp, synth.F16, 1.0 / math.sqrt(d), causal)
    heads = [H - 1]
    ref = pu.run_oracle(inp, synth.F16, 1.0 / math.sqrt(d), causal, heads=heads)
    m = pu.compare(gpu, ref, synth.F16, heads=heads)
    print(f"\n[parity] sweep N={N} d={d} causal={causal} head={heads}: {m}", flush=True)
    pu.assert_within_tolerance(m, ("sweep", d, causal))
